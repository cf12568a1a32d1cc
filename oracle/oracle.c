/*
 * CPU oracle for the per-partition data path of the VIP-caching method: TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, single-threaded C that states what each call of the path computes, written from
 * the paper so that it can be checked against it by eye.  It shares no code with the HIP
 * library and must never be linked, imported or called by it; only the tests, the smoke check
 * and the CPU-baseline leg of the benchmark use it.
 *
 * Conventions (same as the library's interface):
 *   adj(v)  = CSR row v = col[rowptr[v] .. rowptr[v+1])  -- the list v samples its neighbours from
 *   d(v)    = |adj(v)|                                  -- the (outgoing) degree of Sec. 3.1
 *   fanouts[h-1] = f_h, where hop h = 1 is the hop next to the minibatch
 *   [lo,hi) = the owned partition's contiguous id range (Sec. 4.1)
 *
 * Parity pins (tests marked "not gpu"): p^[0] values, range/monotonicity/bound invariants,
 * closed forms on paths and stars, the linear small-probability limit against a library sparse
 * mat-vec, full expansion against boolean frontier expansion, exact enumeration of the random
 * process on graphs of <= 8 vertices, Monte-Carlo frequencies, Philox known-answer vectors,
 * chi-square uniformity of the subset sampler, brute-force sort for the cache ranking.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------------
 * Vertex-inclusion probabilities: Proposition 1, eqs. (1) and (2), with the uniform
 * instantiation given after it: p^[0](u) = B/|T| on T, t_h(u,v) = min(1, f_h/d(v)) if u in adj(v).
 *
 * The product for u runs over every v whose list adj(v) contains u (those are the vertices
 * that can sample u), so it is formed by walking each v's row and multiplying (1 - x_v) into
 * every member u.
 *
 * form = 0: the product is held as a sum of log1p(-x) and p = -expm1(sum); same quantity,
 *           no cancellation for tiny probabilities.
 * form = 1: the literal running product, p = 1 - prod (loses relative accuracy below ~1e-11).
 *
 * p_hop  : double[L*N], p_hop[(h-1)*N + u] = p^[h](u), h = 1..L
 * p_total: double[N],   eq. (1): 1 - prod_{h=1..L}(1 - p^[h](u)); hop 0 multiplied in as well
 *          when include_hop0 != 0.
 * B > |T| clamps p^[0] to 1.  Vertices with d(v) = 0 contribute nothing.
 * verbose != 0 prints one line per finished hop (long runs on 10^9-edge graphs).
 * Returns 0, or -1 on bad arguments / allocation failure.
 * ---------------------------------------------------------------------------------------- */
int orc_vip(int64_t N, const int64_t *rowptr, const int32_t *col, const int32_t *T, int64_t nT,
            int32_t B, const int32_t *fanouts, int32_t L, int include_hop0, int form,
            double *p_hop, double *p_total, int verbose)
{
    if (N <= 0 || L <= 0 || nT <= 0 || B <= 0) return -1;
    double *prev = (double *)calloc((size_t)N, sizeof(double));
    double *acc = (double *)malloc((size_t)N * sizeof(double));  /* product, or sum of logs */
    double *tot = (double *)malloc((size_t)N * sizeof(double));  /* same, over hops */
    if (!prev || !acc || !tot) { free(prev); free(acc); free(tot); return -1; }

    double p0 = (double)B / (double)nT;
    if (p0 > 1.0) p0 = 1.0;
    for (int64_t i = 0; i < nT; ++i) {
        if (T[i] < 0 || T[i] >= N) { free(prev); free(acc); free(tot); return -1; }
        prev[T[i]] = p0;
    }
    for (int64_t u = 0; u < N; ++u) {
        if (form == 0) tot[u] = include_hop0 ? log1p(-prev[u]) : 0.0;
        else           tot[u] = include_hop0 ? 1.0 - prev[u] : 1.0;
    }

    for (int32_t h = 1; h <= L; ++h) {
        double f = (double)fanouts[h - 1];
        for (int64_t u = 0; u < N; ++u) acc[u] = (form == 0) ? 0.0 : 1.0;
        for (int64_t v = 0; v < N; ++v) {
            int64_t d = rowptr[v + 1] - rowptr[v];
            if (d <= 0 || prev[v] <= 0.0) continue;
            double t = f / (double)d;
            if (t > 1.0) t = 1.0;
            double x = t * prev[v];
            double lw = log1p(-x);                 /* the same factor for every member of v's row */
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                int32_t u = col[e];
                if (form == 0) acc[u] += lw;
                else           acc[u] *= (1.0 - x);
            }
        }
        for (int64_t u = 0; u < N; ++u) {
            double ph = (form == 0) ? -expm1(acc[u]) : 1.0 - acc[u];
            p_hop[(int64_t)(h - 1) * N + u] = ph;
            if (form == 0) tot[u] += log1p(-ph);
            else           tot[u] *= (1.0 - ph);
            prev[u] = ph;
        }
        if (verbose) { fprintf(stderr, "[oracle] vip hop %d of %d done\n", h, L); fflush(stderr); }
    }
    for (int64_t u = 0; u < N; ++u)
        p_total[u] = (form == 0) ? -expm1(tot[u]) : 1.0 - tot[u];
    free(prev); free(acc); free(tot);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Cache selection (Sec. 3.2): rank the remote vertices by decreasing score and keep the first
 * C = floor(alpha * N / K).  Ties are broken by ascending id so the set is unique; vertices
 * with score <= 0 are never kept (they are never requested).  The score is compared as the
 * fp32 value the caller passes.  ids_out gets the kept ids in rank order (slot = rank);
 * returns how many were kept (<= C), or -1.
 * ---------------------------------------------------------------------------------------- */
typedef struct { float score; int32_t id; } orc_cand;

static int orc_cand_cmp(const void *a, const void *b)
{
    const orc_cand *x = (const orc_cand *)a, *y = (const orc_cand *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->id > y->id) - (x->id < y->id);
}

int64_t orc_cache_capacity(int64_t N, int32_t K, double alpha)
{
    return (int64_t)floor(alpha * (double)N / (double)K);
}

int64_t orc_cache_select(const float *score, int64_t N, int64_t lo, int64_t hi, int32_t K,
                         double alpha, int32_t *ids_out)
{
    int64_t C = orc_cache_capacity(N, K, alpha);
    orc_cand *c = (orc_cand *)malloc((size_t)(N > 0 ? N : 1) * sizeof(orc_cand));
    if (!c) return -1;
    int64_t n = 0;
    for (int64_t u = 0; u < N; ++u) {
        if (u >= lo && u < hi) continue;         /* local vertices are not cached */
        if (!(score[u] > 0.0f)) continue;
        c[n].score = score[u];
        c[n].id = (int32_t)u;
        ++n;
    }
    qsort(c, (size_t)n, sizeof(orc_cand), orc_cand_cmp);
    int64_t keep = n < C ? n : C;
    for (int64_t i = 0; i < keep; ++i) ids_out[i] = c[i].id;
    free(c);
    return keep;
}

/* ------------------------------------------------------------------------------------------
 * Counter-based random numbers: Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw,
 * "Parallel random numbers: as easy as 1, 2, 3", SC'11), written from the published round
 * function and constants.
 * ---------------------------------------------------------------------------------------- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The draw for (seed, batch, hop, vertex, slot): key = seed (low, high word), counter =
 * (vertex, slot/4, hop, low word of batch), result = word slot%4 of the 128-bit block. */
uint32_t orc_rand32(uint64_t seed, uint64_t batch, uint32_t hop, uint32_t vertex, uint32_t slot)
{
    uint32_t ctr[4] = { vertex, slot >> 2, hop, (uint32_t)batch };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return out[slot & 3u];
}

/* ------------------------------------------------------------------------------------------
 * Node-wise sampling of one vertex (Sec. 2.3, step (ii) of the process in Sec. 3.1): a uniform
 * random subset of min(f, d) positions of adj(v), without replacement.
 * d <= f: every position, in row order, no random numbers.
 * d >  f: Floyd's subset algorithm, one draw per slot j = 0..f-1: with m = d-f+j, t uniform on
 *         [0, m] by multiply-shift of a 32-bit draw; take t unless it was taken, else take m.
 * pos_out gets the positions in slot order; returns their number.
 * ---------------------------------------------------------------------------------------- */
int32_t orc_sample_positions(uint64_t seed, uint64_t batch, uint32_t hop, uint32_t vertex,
                             int64_t d, int32_t f, int64_t *pos_out)
{
    if (d <= f) {
        for (int64_t j = 0; j < d; ++j) pos_out[j] = j;
        return (int32_t)d;
    }
    for (int32_t j = 0; j < f; ++j) {
        uint64_t m = (uint64_t)(d - f + j);
        uint32_t r = orc_rand32(seed, batch, hop, vertex, (uint32_t)j);
        uint64_t t = ((uint64_t)r * (m + 1)) >> 32;
        int taken = 0;
        for (int32_t i = 0; i < j; ++i)
            if ((uint64_t)pos_out[i] == t) { taken = 1; break; }
        pos_out[j] = (int64_t)(taken ? m : t);
    }
    return f;
}

/* ------------------------------------------------------------------------------------------
 * Multi-hop sampling into per-layer message-flow graphs.
 * S_0 = seeds.  At hop h every vertex of S_{h-1}, in order, samples with fanout f_h; the
 * sampled ids are laid out target-major, slot-minor.  S_h = S_{h-1} followed by the ids not
 * seen before, in order of first appearance.  MFG h: indptr[h-1] (n_{h-1}+1 offsets) and
 * src[h-1] (local index in S_h of every sampled id).
 *
 * node_ids: int32[node_cap]; indptr[h-1]: int32[>= n_{h-1}+1]; src[h-1]: int32[edge_cap];
 * n_out, e_out: int64[L+1] (n_out[0] = nseeds, e_out[0] = 0).
 * Returns 0; -1 bad args/alloc; -2 capacity exceeded.
 * ---------------------------------------------------------------------------------------- */
int orc_sample_mfg(int64_t N, const int64_t *rowptr, const int32_t *col, const int32_t *seeds,
                   int32_t nseeds, const int32_t *fanouts, int32_t L, uint64_t seed, uint64_t batch,
                   int64_t node_cap, int64_t edge_cap, int32_t *node_ids, int32_t **indptr,
                   int32_t **src, int64_t *n_out, int64_t *e_out)
{
    if (N <= 0 || nseeds < 0 || L <= 0 || nseeds > node_cap) return -1;
    int32_t *local = (int32_t *)malloc((size_t)N * sizeof(int32_t));   /* global id -> index in S */
    if (!local) return -1;
    for (int64_t g = 0; g < N; ++g) local[g] = -1;
    int64_t n = 0;
    for (int32_t i = 0; i < nseeds; ++i) {
        int32_t g = seeds[i];
        if (g < 0 || g >= N || local[g] >= 0) { free(local); return -1; }   /* distinct, in range */
        local[g] = (int32_t)n;
        node_ids[n++] = g;
    }
    n_out[0] = n; e_out[0] = 0;
    int rc = 0;
    for (int32_t h = 1; h <= L && rc == 0; ++h) {
        int32_t f = fanouts[h - 1];
        int64_t *pos = (int64_t *)malloc((size_t)(f > 0 ? f : 1) * sizeof(int64_t));
        if (!pos) { rc = -1; break; }
        int64_t n_prev = n, e = 0;
        int32_t *ip = indptr[h - 1], *sp = src[h - 1];
        for (int64_t i = 0; i < n_prev && rc == 0; ++i) {
            int32_t v = node_ids[i];
            int64_t d = rowptr[v + 1] - rowptr[v];
            ip[i] = (int32_t)e;
            int32_t c = orc_sample_positions(seed, batch, (uint32_t)h, (uint32_t)v, d, f, pos);
            for (int32_t j = 0; j < c; ++j) {
                int32_t g = col[rowptr[v] + pos[j]];
                if (local[g] < 0) {
                    if (n >= node_cap) { rc = -2; break; }
                    local[g] = (int32_t)n;
                    node_ids[n++] = g;
                }
                if (e >= edge_cap) { rc = -2; break; }
                sp[e++] = local[g];
            }
        }
        ip[n_prev] = (int32_t)e;
        n_out[h] = n; e_out[h] = e;
        free(pos);
    }
    free(local);
    return rc;
}

/* ------------------------------------------------------------------------------------------
 * Cache-aware feature gather (Secs. 4.1-4.3): out[i,:] = X[node_ids[i],:], where row g of the
 * conceptual matrix X lives in exactly one of three stores:
 *   local  [hi-lo rows]   if lo <= g < hi          (row g - lo)
 *   cache  [n_cached rows] if g is in cache_ids     (row = its rank/slot)
 *   remote [N-(hi-lo) rows] otherwise               (row g if g < lo else g - (hi-lo))
 * Cache rows are copies of remote rows, so the source never changes a byte of the result.
 * src_tag (optional): 0 local, 1 cache, 2 remote miss.  counts: n_local, n_cache_hit, n_miss.
 * ---------------------------------------------------------------------------------------- */
int orc_gather(int64_t N, int64_t lo, int64_t hi, const void *local, const void *cache,
               const int32_t *cache_ids, int64_t n_cached, const void *remote, int64_t row_bytes,
               const int32_t *node_ids, int64_t n, void *out, int8_t *src_tag, int64_t counts[3])
{
    int32_t *slot = (int32_t *)malloc((size_t)N * sizeof(int32_t));
    if (!slot) return -1;
    for (int64_t g = 0; g < N; ++g) slot[g] = -1;
    for (int64_t s = 0; s < n_cached; ++s) slot[cache_ids[s]] = (int32_t)s;
    counts[0] = counts[1] = counts[2] = 0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t g = node_ids[i];
        if (g < 0 || g >= N) { free(slot); return -1; }
        const char *from;
        int tag;
        if (g >= lo && g < hi)   { from = (const char *)local + (g - lo) * row_bytes; tag = 0; }
        else if (slot[g] >= 0)   { from = (const char *)cache + (int64_t)slot[g] * row_bytes; tag = 1; }
        else { int64_t r = g < lo ? g : g - (hi - lo);
               from = (const char *)remote + r * row_bytes; tag = 2; }
        memcpy((char *)out + i * row_bytes, from, (size_t)row_bytes);
        if (src_tag) src_tag[i] = (int8_t)tag;
        counts[tag]++;
    }
    free(slot);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * VIP-ordered local storage (Sec. 3.2, paragraph on host-to-device transfer reduction; Sec. 4.1;
 * the experiment of Sec. 5 on local partition storage on CPU versus GPU): the partition's own
 * vertices are ranked by decreasing score, and the features of the first floor(beta * (hi-lo))
 * of that order are kept in device memory; the others stay in host memory.
 * Order: score descending, vertex id ascending among equal scores; a score that is not
 * positive (or not a number) counts as 0.  A constant score therefore gives the id order
 * (the "no reorder" baseline of that experiment).
 *   rank[i]  = position of local vertex lo + i in the order
 *   order[r] = local index of the vertex at position r
 * ---------------------------------------------------------------------------------------- */
int64_t orc_local_capacity(double beta, int64_t n_local)
{
    if (!(beta > 0.0)) return 0;
    double c = floor(beta * (double)n_local);
    if (c > (double)n_local) c = (double)n_local;
    return (int64_t)c;
}

typedef struct { float s; int32_t i; } orc_local_item;

static int orc_local_cmp(const void *a, const void *b)
{
    const orc_local_item *x = (const orc_local_item *)a, *y = (const orc_local_item *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

int orc_local_rank(const float *score, int64_t lo, int64_t hi, int32_t *rank, int32_t *order)
{
    const int64_t n = hi - lo;
    if (n <= 0) return 0;
    orc_local_item *it = (orc_local_item *)malloc((size_t)n * sizeof(orc_local_item));
    if (!it) return -1;
    for (int64_t i = 0; i < n; ++i) {
        const float s = score[lo + i];
        it[i].s = (s > 0.0f) ? s : 0.0f;          /* false for NaN too */
        it[i].i = (int32_t)i;
    }
    qsort(it, (size_t)n, sizeof(orc_local_item), orc_local_cmp);
    for (int64_t r = 0; r < n; ++r) {
        order[r] = it[r].i;
        rank[it[r].i] = (int32_t)r;
    }
    free(it);
    return 0;
}

/* The gather of orc_gather with the local store split in two:
 *   local_dev  [n_dev rows]   rows of the first n_dev vertices of the order (row = rank)
 *   local_host [hi-lo rows]   all local rows in id order (row g - lo); read for rank >= n_dev
 * src_tag: 0 local from device, 1 cache, 2 remote miss, 3 local from host.
 * counts: the same four, in that order.  The split never changes a byte of the result. */
int orc_gather_split(int64_t N, int64_t lo, int64_t hi, const void *local_dev, const void *local_host,
                     const int32_t *rank, int64_t n_dev, const void *cache, const int32_t *cache_ids,
                     int64_t n_cached, const void *remote, int64_t row_bytes, const int32_t *node_ids,
                     int64_t n, void *out, int8_t *src_tag, int64_t counts[4])
{
    int32_t *slot = (int32_t *)malloc((size_t)N * sizeof(int32_t));
    if (!slot) return -1;
    for (int64_t g = 0; g < N; ++g) slot[g] = -1;
    for (int64_t s = 0; s < n_cached; ++s) slot[cache_ids[s]] = (int32_t)s;
    counts[0] = counts[1] = counts[2] = counts[3] = 0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t g = node_ids[i];
        if (g < 0 || g >= N) { free(slot); return -1; }
        const char *from;
        int tag;
        if (g >= lo && g < hi) {
            const int64_t r = rank[g - lo];
            if (r < n_dev) { from = (const char *)local_dev + r * row_bytes; tag = 0; }
            else           { from = (const char *)local_host + (g - lo) * row_bytes; tag = 3; }
        }
        else if (slot[g] >= 0)   { from = (const char *)cache + (int64_t)slot[g] * row_bytes; tag = 1; }
        else { int64_t r = g < lo ? g : g - (hi - lo);
               from = (const char *)remote + r * row_bytes; tag = 2; }
        memcpy((char *)out + i * row_bytes, from, (size_t)row_bytes);
        if (src_tag) src_tag[i] = (int8_t)tag;
        counts[tag]++;
    }
    free(slot);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Empirical access frequencies (Sec. 3.2, the "sim." and "oracle" caching policies): count[v] is
 * the number of minibatches whose sampled vertex set S_L contains v.  "sim." counts over simulated
 * epochs before training, "oracle" over the epochs that are evaluated; either count is then ranked
 * exactly like a VIP score.  One call adds one id list (ids of a minibatch are distinct, so a
 * vertex gains at most 1 per minibatch; a repeated id would count every time it appears).
 * ---------------------------------------------------------------------------------------- */
int orc_access_count(int64_t N, const int32_t *node_ids, int64_t n, float *count)
{
    for (int64_t i = 0; i < n; ++i) {
        const int64_t g = node_ids[i];
        if (g < 0 || g >= N) return -1;
        count[g] += 1.0f;
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Proposition 1 with arbitrary initial and transition probabilities (Sec. 3.1, the paragraph
 * after the proposition: any initial sampling, any hop-wise transition probability function):
 *   p0[v]     probability that v is in the minibatch                         (float32[N])
 *   t[h-1][e] probability that the vertex of CSR row r(e) samples col[e] at hop h  (float32[M])
 *   p^[h](u) = 1 - prod over edges e with col[e] = u of (1 - t[h-1][e] * p^[h-1](r(e)))   eq. (2)
 *   p(u)     = 1 - prod_{h=1..L} (1 - p^[h](u))                                          eq. (1)
 * Products are carried as fp64 sums of log1p.  Every probability must lie in [0, 1].
 * include_hop0 multiplies (1 - p0) into eq. (1), as for the uniform instantiation.
 * p_hop: double[L*N] or NULL; p_total: double[N].  Returns 0; -1 bad argument; -3 a value
 * outside [0, 1] (or not a number).
 * ---------------------------------------------------------------------------------------- */
int orc_vip_general(int64_t N, const int64_t *rowptr, const int32_t *col, const float *p0,
                    const float *const *t, int32_t L, int include_hop0, double *p_hop, double *p_total)
{
    if (N <= 0 || L <= 0 || !p0 || !t || !p_total) return -1;
    const int64_t M = rowptr[N];
    for (int64_t v = 0; v < N; ++v)
        if (!(p0[v] >= 0.0f && p0[v] <= 1.0f)) return -3;
    for (int32_t h = 0; h < L; ++h)
        for (int64_t e = 0; e < M; ++e)
            if (!(t[h][e] >= 0.0f && t[h][e] <= 1.0f)) return -3;
    double *prev = (double *)malloc((size_t)N * sizeof(double));
    double *S = (double *)malloc((size_t)N * sizeof(double));
    double *tot = (double *)calloc((size_t)N, sizeof(double));
    if (!prev || !S || !tot) { free(prev); free(S); free(tot); return -1; }
    for (int64_t v = 0; v < N; ++v) {
        prev[v] = (double)p0[v];
        if (include_hop0) tot[v] = log1p(-prev[v]);
    }
    for (int32_t h = 1; h <= L; ++h) {
        for (int64_t u = 0; u < N; ++u) S[u] = 0.0;
        for (int64_t v = 0; v < N; ++v) {
            if (prev[v] == 0.0) continue;
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                const double x = (double)t[h - 1][e] * prev[v];
                if (x > 0.0) S[col[e]] += log1p(-x);
            }
        }
        for (int64_t u = 0; u < N; ++u) {
            prev[u] = -expm1(S[u]);
            tot[u] += S[u];
            if (p_hop) p_hop[(int64_t)(h - 1) * N + u] = prev[u];
        }
    }
    for (int64_t u = 0; u < N; ++u) p_total[u] = -expm1(tot[u]);
    free(prev); free(S); free(tot);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * A sampler whose transition probabilities are exactly t: at hop h a target v takes every member
 * col[e] of its row independently with probability t[h-1][e] (independent inclusion, so a
 * target's sample has no fixed size).  Edge e at position k of its row is taken iff
 *   rand32(seed, batch, h, v, k) < floor(t[h-1][e] * 2^32)      (compared as 64-bit integers),
 * so the realised probability is t rounded down to a multiple of 2^-32, and t = 1 always takes.
 * Layout and relabelling as in orc_sample_mfg: taken neighbours of a target in row order,
 * targets in the order of S_{h-1}, new ids appended in order of first appearance.
 * With node_ids == NULL only the sizes n_out, e_out are computed (to size the buffers).
 * Returns 0; -1 bad args/alloc; -2 capacity exceeded.
 * ---------------------------------------------------------------------------------------- */
int orc_sample_mfg_general(int64_t N, const int64_t *rowptr, const int32_t *col, const float *const *t,
                           const int32_t *seeds, int32_t nseeds, int32_t L, uint64_t seed, uint64_t batch,
                           int64_t node_cap, int64_t edge_cap, int32_t *node_ids, int32_t **indptr,
                           int32_t **src, int64_t *n_out, int64_t *e_out)
{
    if (N <= 0 || nseeds < 0 || L <= 0) return -1;
    const int count_only = node_ids == NULL;
    int32_t *local = (int32_t *)malloc((size_t)N * sizeof(int32_t));   /* global id -> index in S */
    int32_t *S = (int32_t *)malloc((size_t)N * sizeof(int32_t));       /* S_h (at most N ids) */
    if (!local || !S) { free(local); free(S); return -1; }
    for (int64_t g = 0; g < N; ++g) local[g] = -1;
    int64_t n = 0;
    for (int32_t i = 0; i < nseeds; ++i) {
        int32_t g = seeds[i];
        if (g < 0 || g >= N || local[g] >= 0) { free(local); free(S); return -1; }
        local[g] = (int32_t)n;
        S[n++] = g;
    }
    n_out[0] = n; e_out[0] = 0;
    int rc = 0;
    for (int32_t h = 1; h <= L && rc == 0; ++h) {
        const int64_t n_prev = n;
        int64_t e = 0;
        int32_t *ip = count_only ? NULL : indptr[h - 1], *sp = count_only ? NULL : src[h - 1];
        for (int64_t i = 0; i < n_prev && rc == 0; ++i) {
            const int32_t v = S[i];
            if (ip) ip[i] = (int32_t)e;
            for (int64_t k = 0; k < rowptr[v + 1] - rowptr[v]; ++k) {
                const int64_t edge = rowptr[v] + k;
                const uint64_t thr = (uint64_t)((double)t[h - 1][edge] * 4294967296.0);
                const uint32_t r = orc_rand32(seed, batch, (uint32_t)h, (uint32_t)v, (uint32_t)k);
                if (!((uint64_t)r < thr)) continue;
                const int32_t g = col[edge];
                if (local[g] < 0) { local[g] = (int32_t)n; S[n++] = g; }
                if (sp) {
                    if (e >= edge_cap) { rc = -2; break; }
                    sp[e] = local[g];
                }
                ++e;
            }
        }
        if (ip) ip[n_prev] = (int32_t)e;
        n_out[h] = n; e_out[h] = e;
    }
    if (!count_only && rc == 0) {
        if (n > node_cap) rc = -2;
        else memcpy(node_ids, S, (size_t)n * sizeof(int32_t));
    }
    free(local); free(S);
    return rc;
}
