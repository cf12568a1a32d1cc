// Vertex-inclusion probabilities, Proposition 1 (Sec. 3.1), in pull form over row blocks.
//
// Per hop h every vertex v carries y_h(v) = log1p(-x_h(v)), x_h(v) = min(1, f_h/d(v)) * p^[h-1](v)
// (0 for d(v) = 0), stored as fp32.  Then eq. (2) is
//     S_h(u) = sum over {v : u in adj(v)} of y_h(v)     (all terms <= 0: no cancellation; fp64 sums)
//     p^[h](u) = -expm1(S_h(u))
// and because log(1 - p^[h](u)) = S_h(u), eq. (1) is p(u) = -expm1(sum_h S_h(u)).
//
// Dense hops: the edges are stored grouped by blocks of 2^14 destination rows and sorted by source
// inside a block.  A workgroup keeps the block's fp64 sums in LDS (128 KB), streams a share of the
// block's edges (4 bytes each, read as 128-bit vectors) and adds y[source] to the row's sum with an
// LDS atomic; because the sources ascend, neighbouring lanes gather from neighbouring lines of y and
// a line fetched from L2 serves every edge of the block that needs it.  (A pull that walks one
// row's in-list at a time fetches a line per edge: it ran at a third of this rate on every graph
// measured, from 2.4M to 134M vertices.)  A second kernel adds the shares and finishes the vertex
// (p^[h], running total, next hop's y).
//
// Early hops touch few edges (hop 1 only the rows of T), so the kernel that writes a hop's y also
// counts the hop's frontier (vertices with y != 0) and its out-edges; when that is a small share of
// the graph the frontier is compacted into a list and the hop is done in push form instead: each
// frontier vertex adds its y to the fp64 accumulator of every member of its row (atomic adds), and
// one pass finishes all vertices.
#include "spp_common.h"
#include "spp_device.h"

namespace spp {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int64_t kPushShare = 16;       // push when the frontier's out-edges are at most M/16
constexpr int kStatBlocks = 2048;        // most workgroups that report a part of the next frontier's size
constexpr int kStatMirror = 2048;        // where those reports land in the context's pinned mirror (int64 index)

struct VipHop {
    const int64_t* rowptr;     // forward CSR, for d(u)
    const float*   y;          // this hop's y
    float*         y_next;     // next hop's y (unused at the last hop)
    double*        tot;        // running sum of S over hops
    float*         p_hop;      // p^[h] or null
    float*         p_total;    // written at the last hop
    double         f_next;     // f_{h+1}
    int            first;      // first hop and hop 0 not included: tot is not read
    int            last;
    unsigned long long* stat;  // per workgroup: vertices and out-edges of the next hop's frontier (unused at the last hop)
};

// `told` = the running total read beforehand (ignored at a first hop).
__device__ __forceinline__ void vip_finish_vertex(const VipHop& a, int64_t u, double S, double told,
                                                  unsigned long long& verts, unsigned long long& edges) {
    // A vertex that no frontier vertex points at has S = 0 exactly (most vertices, at the early hops):
    // its p^[h] is 0 and it needs no exponential; nor does p^[h] at the last hop when it is not asked for.
    const bool need_ph = a.p_hop != nullptr || !a.last;
    const double ph = (need_ph && S != 0.0) ? -expm1(S) : 0.0;
    if (a.p_hop) a.p_hop[u] = (float)ph;
    const double T = a.first ? S : told + S;
    if (a.last) {
        a.p_total[u] = T != 0.0 ? (float)(-expm1(T)) : 0.0f;
    } else {
        a.tot[u] = T;
        float yn = 0.f;
        if (ph > 0.0) {
            const int64_t d = a.rowptr[u + 1] - a.rowptr[u];
            if (d > 0) {
                double t = a.f_next / (double)d;
                if (t > 1.0) t = 1.0;
                yn = (float)log1p(-(t * ph));
                if (yn != 0.0f) { ++verts; edges += (unsigned long long)d; }
            }
        }
        a.y_next[u] = yn;
    }
}

__device__ __forceinline__ void vip_finish_vertex(const VipHop& a, int64_t u, double S, unsigned long long& verts,
                                                  unsigned long long& edges) {
    vip_finish_vertex(a, u, S, a.first ? 0.0 : a.tot[u], verts, edges);
}
// All vertices, grid-stride, four per thread and round: the four sums and running totals are in
// flight together (one vertex per round leaves a pass over 10^8 vertices waiting on its own loads:
// 0.87 ms where the bytes take 0.55).  sum_of(u) = S_h(u).
template <class SumOf>
__device__ __forceinline__ void vip_finish_all(const VipHop& a, int64_t N, SumOf sum_of, unsigned long long& verts,
                                               unsigned long long& edges) {
    constexpr int U = 4;
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    for (; u + (U - 1) * stride < N; u += U * stride) {
        double S[U], T0[U];
#pragma unroll
        for (int k = 0; k < U; ++k) S[k] = sum_of(u + k * stride);
#pragma unroll
        for (int k = 0; k < U; ++k) T0[k] = a.first ? 0.0 : a.tot[u + k * stride];
#pragma unroll
        for (int k = 0; k < U; ++k) vip_finish_vertex(a, u + k * stride, S[k], T0[k], verts, edges);
    }
    for (; u < N; u += stride) vip_finish_vertex(a, u, sum_of(u), verts, edges);
}

// The next hop is pushed or pulled depending on the size of its frontier (vertices with y != 0 and
// their out-edges); the kernel that writes the next hop's y counts both on the way, one pair per
// workgroup (no atomics: same-address atomics cost about 15 ns each), and the host adds the pairs.
__device__ __forceinline__ void write_frontier_stat(unsigned long long* stat, unsigned long long verts,
                                                    unsigned long long edges) {
    __shared__ unsigned long long red[2][kBlock / kWave];
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        verts += __shfl_down((long long)verts, off, kWave);
        edges += __shfl_down((long long)edges, off, kWave);
    }
    if (lane_id() == 0) { red[0][threadIdx.x >> 6] = verts; red[1][threadIdx.x >> 6] = edges; }
    __syncthreads();
    if (threadIdx.x == 0) {
        stat[2 * blockIdx.x] = red[0][0] + red[0][1] + red[0][2] + red[0][3];
        stat[2 * blockIdx.x + 1] = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    }
}

__global__ void fill_f32_kernel(float* p, int64_t n, float v) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}
__global__ void fill_f64_kernel(double* p, int64_t n, double v) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if ((reinterpret_cast<uintptr_t>(p) & 15) == 0) {        // 128-bit stores for the bulk
        typedef double f64x2 __attribute__((ext_vector_type(2)));
        const f64x2 vv = {v, v};
        f64x2* p2 = reinterpret_cast<f64x2*>(p);
        for (int64_t i = tid; i < (n >> 1); i += stride) p2[i] = vv;
        if (tid == 0 && (n & 1)) p[n - 1] = v;
        return;
    }
    for (int64_t i = tid; i < n; i += stride) p[i] = v;
}

// The frontier itself (any order): list[0 .. *cursor) = vertices whose y is not zero and whose row
// is not empty; a row of more than kPieceEdges entries is listed once per piece of that many
// entries (adjacent in the list), so that the kernels that walk the frontier's rows can hand the
// pieces of a long row to different workgroups.  A thread looks at kListPer vertices (as 128-bit vectors),
// first to count its entries and, once the workgroup has reserved its part of the list with one
// atomic, again to write them (the second look finds its lines in the caches).  Same-address
// atomics cost about 15 ns each, so what a round covers sets the pace on a large graph: with 8
// vertices per thread a dense frontier of 10^8 vertices took 0.72 ms (54k atomics), with 64 the
// pass is bound by reading y.  Small graphs keep 8 per thread (enough workgroups to fill the chip).
constexpr int64_t kPieceEdges = 4096;
__host__ __device__ inline int64_t frontier_list_capacity(int64_t N, int64_t M) { return N + M / kPieceEdges; }

template <int kListPer>
__global__ void __launch_bounds__(kBlock) vip_frontier_list_kernel(const float* __restrict__ y,
                                                                   const int64_t* __restrict__ rowptr, int64_t N,
                                                                   int32_t* __restrict__ list,
                                                                   unsigned long long* __restrict__ cursor) {
    __shared__ int scan_lds[4];
    __shared__ unsigned long long start;
    const int64_t round = (int64_t)kBlock * kListPer;
    auto pieces = [&](int64_t v) { return (int)((rowptr[v + 1] - rowptr[v] + kPieceEdges - 1) / kPieceEdges); };
    for (int64_t r0 = (int64_t)blockIdx.x * round; r0 < N; r0 += (int64_t)gridDim.x * round) {
        // A wavefront covers kWave * kListPer consecutive vertices; lane l takes the 128-bit vectors
        // l, 64 + l, 128 + l, ... of them (whole lines per load).  Bit 4 k + c of nz: component c of the
        // lane's k-th vector is in the frontier.  (y is 16-byte aligned and w0 a multiple of four.)
        const int64_t w0 = r0 + (int64_t)(threadIdx.x >> 6) * (kWave * kListPer);
        auto vertex = [&](int bit) { return w0 + 4 * ((int64_t)(bit >> 2) * kWave + lane_id()) + (bit & 3); };
        uint64_t nz = 0;
#pragma unroll
        for (int k = 0; k < kListPer / 4; ++k) {
            const int64_t v = vertex(4 * k);
            if (v + 3 < N) {
                const f32x4 t = *reinterpret_cast<const f32x4*>(y + v);
                nz |= (uint64_t)((t.x != 0.0f) | ((t.y != 0.0f) << 1) | ((t.z != 0.0f) << 2) | ((t.w != 0.0f) << 3)) << (4 * k);
            } else {
                for (int c = 0; c < 4; ++c)
                    if (v + c < N && y[v + c] != 0.0f) nz |= 1ull << (4 * k + c);
            }
        }
        int mine = 0;
        for (uint64_t m = nz; m; m &= m - 1) mine += pieces(vertex(__builtin_ctzll(m)));
        int total;
        int at = block_exclusive_scan(mine, scan_lds, total);
        if (total == 0) continue;        // uniform over the workgroup: the scan has synchronised it
        if (threadIdx.x == 0) start = atomicAdd(cursor, (unsigned long long)total);
        __syncthreads();
        const unsigned long long base = start;
        for (uint64_t m = nz; m; m &= m - 1) {
            const int64_t v = vertex(__builtin_ctzll(m));
            for (int c = pieces(v); c > 0; --c) list[base + at++] = (int32_t)v;
        }
        __syncthreads();
    }
}

inline void launch_frontier_list(int grid, hipStream_t st, const float* y, const int64_t* rowptr, int64_t N, int32_t* list,
                                 unsigned long long* cursor) {
    if (N >= (int64_t)1 << 25) vip_frontier_list_kernel<64><<<grid, kBlock, 0, st>>>(y, rowptr, N, list, cursor);
    else vip_frontier_list_kernel<8><<<grid, kBlock, 0, st>>>(y, rowptr, N, list, cursor);
}

// Entry i of that list: where its piece of the row starts in col[] and how many entries it has.
// The pieces of a row are adjacent and in order, so the number of the piece is the distance to
// the first entry with the same vertex (found by galloping, then bisection).
__device__ __forceinline__ int32_t frontier_entry(const int32_t* __restrict__ list, int64_t i,
                                                  const int64_t* __restrict__ rowptr, int64_t& row, uint32_t& deg) {
    const int32_t v = list[i];
    int64_t lo = i, step = 1;                               // list[lo] == v
    while (lo - step >= 0 && list[lo - step] == v) { lo -= step; step <<= 1; }
    int64_t a = lo - step < 0 ? -1 : lo - step;             // a == -1 or list[a] != v
    while (lo - a > 1) {
        const int64_t mid = (a + lo) >> 1;
        if (list[mid] == v) lo = mid; else a = mid;
    }
    const int64_t b = rowptr[v] + (i - lo) * kPieceEdges, e = rowptr[v + 1];
    row = b;
    deg = (uint32_t)(e - b < kPieceEdges ? e - b : kPieceEdges);
    return v;
}

__global__ void __launch_bounds__(kBlock) vip_push_finish_kernel(VipHop a, const double* __restrict__ acc, int64_t N) {
    unsigned long long verts = 0, edges = 0;
    vip_finish_all(a, N, [&](int64_t u) { return acc[u]; }, verts, edges);
    if (!a.last) write_frontier_stat(a.stat, verts, edges);
}

// Dense hops, blocked: one workgroup takes the j-th of `parts` equal shares of the edges that end
// in one block of 2^rbits destination rows.  The block's fp64 sums live in LDS; the edges are
// sorted by source, so the gathers of y sweep the vector once, neighbouring lanes read
// neighbouring lines, and a line fetched from L2 serves every edge of the block that needs it
// (in a row-ordered pull every edge fetches a line of its own).  The share's sums are written
// to part[j][row]; the finish kernel adds the shares.
// An edge is one 32-bit word (low 18 bits of the source, row inside the block); the source's high
// bits follow from the edge's position: the block's chunk bounds sit in LDS next to the sums, a
// lane finds the chunk of the first of its four consecutive edges by bisection and steps forward
// for the other three.
constexpr int kTileBlock = 1024;
constexpr int kTileUnroll = 2;          // 128-bit vectors (four edges) per lane and round
__global__ void __launch_bounds__(kTileBlock) vip_tile_kernel(const uint32_t* __restrict__ t_edge,
                                                              const int64_t* __restrict__ first, int nch, int parts,
                                                              int rbits, const float* __restrict__ y,
                                                              double* __restrict__ part, int64_t part_stride) {
    extern __shared__ double acc[];
    const int R = 1 << rbits;
    uint32_t* bound = reinterpret_cast<uint32_t*>(acc + R);
    // share-major order: the workgroups that run at the same time take the same share of different
    // blocks, i.e. the same part of y (block-major order: 228 us instead of 214)
    const int64_t nrb = gridDim.x / parts;
    const int64_t rb = blockIdx.x % nrb;
    const int j = (int)(blockIdx.x / nrb);
    const int64_t b0 = first[rb * nch], len = first[(rb + 1) * nch] - b0;
    for (int i = threadIdx.x; i < R; i += kTileBlock) acc[i] = 0.0;
    for (int c = threadIdx.x; c <= nch; c += kTileBlock) bound[c] = (uint32_t)(first[rb * nch + c] - b0);
    __syncthreads();
    const int64_t beg = b0 + len * j / parts, end = b0 + len * (j + 1) / parts;
    // The edge stream is read four edges per lane (one 128-bit load): a CU keeps a limited number
    // of misses in flight, so the bytes per request decide the streaming rate.  Software pipeline:
    // the words of the next round are in flight while this round's gathers and LDS adds run.
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    int64_t a4 = (beg + 3) & ~(int64_t)3, e4 = end & ~(int64_t)3;
    if (a4 > end) a4 = end;
    if (e4 < a4) e4 = a4;
    auto one = [&](int64_t e) {
        const uint32_t w = t_edge[e];
        const float v = y[tile_source(w, tile_chunk_of(bound, nch, (uint32_t)(e - b0)))];
        if (v != 0.0f) unsafeAtomicAdd(&acc[w & kTileRowMask], (double)v);
    };
    for (int64_t e = beg + threadIdx.x; e < a4; e += kTileBlock) one(e);      // unaligned head
    for (int64_t e = e4 + threadIdx.x; e < end; e += kTileBlock) one(e);      // tail
    const u32x4* __restrict__ vs = reinterpret_cast<const u32x4*>(t_edge + a4);
    const int64_t nvec = (e4 - a4) >> 2;
    const uint32_t p0 = (uint32_t)(a4 - b0);                                   // position of the first vector's first edge
    constexpr int64_t kRound = (int64_t)kTileUnroll * kTileBlock;
    u32x4 s[kTileUnroll];
    int ch[kTileUnroll];                 // chunk of the lane's current vector and where that chunk ends;
    uint32_t ch_end[kTileUnroll];        // a lane's positions only grow, so both only move forward
    int64_t q = threadIdx.x;
#pragma unroll
    for (int u = 0; u < kTileUnroll; ++u) {
        ch[u] = 0; ch_end[u] = 0;
        if (q + u * kTileBlock < nvec) {
            s[u] = __builtin_nontemporal_load(vs + q + u * kTileBlock);
            ch[u] = tile_chunk_of(bound, nch, p0 + 4u * (uint32_t)(q + u * kTileBlock));
            ch_end[u] = bound[ch[u] + 1];
        }
    }
    for (; q < nvec; q += kRound) {
        u32x4 sn[kTileUnroll];
#pragma unroll
        for (int u = 0; u < kTileUnroll; ++u)
            if (q + kRound + u * kTileBlock < nvec) sn[u] = __builtin_nontemporal_load(vs + q + kRound + u * kTileBlock);
        float v[kTileUnroll][4];
#pragma unroll
        for (int u = 0; u < kTileUnroll; ++u)
            if (q + u * kTileBlock < nvec) {
                const uint32_t p = p0 + 4u * (uint32_t)(q + u * kTileBlock);
                int c = ch[u];
                uint32_t ce = ch_end[u];
                while (p >= ce) { ++c; ce = bound[c + 1]; }      // p + 3 < len = bound[nch]: c stays below nch
                if (p + 3 < ce) {                                  // the four edges share a chunk
                    v[u][0] = y[tile_source(s[u].x, c)];
                    v[u][1] = y[tile_source(s[u].y, c)];
                    v[u][2] = y[tile_source(s[u].z, c)];
                    v[u][3] = y[tile_source(s[u].w, c)];
                } else {
                    v[u][0] = y[tile_source(s[u].x, c)];
                    while (p + 1 >= ce) { ++c; ce = bound[c + 1]; }
                    v[u][1] = y[tile_source(s[u].y, c)];
                    while (p + 2 >= ce) { ++c; ce = bound[c + 1]; }
                    v[u][2] = y[tile_source(s[u].z, c)];
                    while (p + 3 >= ce) { ++c; ce = bound[c + 1]; }
                    v[u][3] = y[tile_source(s[u].w, c)];
                }
                ch[u] = c; ch_end[u] = ce;
            }
#pragma unroll
        for (int u = 0; u < kTileUnroll; ++u)
            if (q + u * kTileBlock < nvec) {
                if (v[u][0] != 0.0f) unsafeAtomicAdd(&acc[s[u].x & kTileRowMask], (double)v[u][0]);
                if (v[u][1] != 0.0f) unsafeAtomicAdd(&acc[s[u].y & kTileRowMask], (double)v[u][1]);
                if (v[u][2] != 0.0f) unsafeAtomicAdd(&acc[s[u].z & kTileRowMask], (double)v[u][2]);
                if (v[u][3] != 0.0f) unsafeAtomicAdd(&acc[s[u].w & kTileRowMask], (double)v[u][3]);
            }
#pragma unroll
        for (int u = 0; u < kTileUnroll; ++u) s[u] = sn[u];
    }
    __syncthreads();
    double* __restrict__ out = part + (int64_t)j * part_stride + (rb << rbits);
    for (int i = threadIdx.x; i < R; i += kTileBlock) out[i] = acc[i];
}

__global__ void __launch_bounds__(kBlock) vip_tile_finish_kernel(VipHop a, const double* __restrict__ part, int parts,
                                                                 int64_t part_stride, int64_t N) {
    unsigned long long verts = 0, edges = 0;
    vip_finish_all(a, N, [&](int64_t u) {
        double S = part[u];
        for (int j = 1; j < parts; ++j) S += part[(int64_t)j * part_stride + u];
        return S;
    }, verts, edges);
    if (!a.last) write_frontier_stat(a.stat, verts, edges);
}

// ---- dense hops over the chunked layout -------------------------------------------------------
// When y does not stay in the caches (10^8 vertices: 444 MB), the gathers of the kernel above fetch
// a 128-byte line per edge and the hop runs at a tenth of the edge stream's rate.  The chunked
// layout trades bytes for order.  First pass: one workgroup per chunk of 2^15 sources keeps the
// chunk's y in LDS (128 KB) and writes y[source] for every entry of the chunk, in entry order:
// 2 bytes read and 4 written per entry, all of it streamed.  Second pass: one workgroup per row
// block keeps the block's fp64 sums in LDS and adds up the block's pieces, one from every chunk
// (4 + 2 bytes read per entry in runs of about a hundred entries, found through two tables that are
// staged in LDS 2048 pieces at a time), then finishes the block's vertices itself.  12 bytes per
// entry instead of 4, but no line is fetched for four of its bytes.
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));
constexpr int kXBlock = 1024;
constexpr int kXUnroll = 4;              // vectors (four entries) per lane and round of the first pass (2, 4, 8: the same time)

__global__ void __launch_bounds__(kXBlock) vip_expand_kernel(const uint16_t* __restrict__ x_src,
                                                             const int64_t* __restrict__ chunk_first, int nch, int64_t N,
                                                             const float* __restrict__ y, float* __restrict__ vals) {
    extern __shared__ float ych[];
    constexpr int C = 1 << kXSrcBits;
    for (int c = blockIdx.x; c < nch; c += gridDim.x) {
        const int64_t v0 = (int64_t)c << kXSrcBits;
        int any = 0;
        if (v0 + C <= N) {               // y is 16-byte aligned and v0 a multiple of C
            const f32x4* __restrict__ y4 = reinterpret_cast<const f32x4*>(y + v0);
            f32x4 t[C / 4 / kXBlock];
#pragma unroll
            for (int k = 0; k < C / 4 / kXBlock; ++k) t[k] = y4[threadIdx.x + k * kXBlock];
#pragma unroll
            for (int k = 0; k < C / 4 / kXBlock; ++k) {
                reinterpret_cast<f32x4*>(ych)[threadIdx.x + k * kXBlock] = t[k];
                any |= (t[k].x != 0.0f) | (t[k].y != 0.0f) | (t[k].z != 0.0f) | (t[k].w != 0.0f);
            }
        } else {
            for (int i = threadIdx.x; i < C; i += kXBlock) {
                const float t = v0 + i < N ? y[v0 + i] : 0.0f;
                ych[i] = t;
                any |= t != 0.0f;
            }
        }
        if (threadIdx.x == 0) ych[C] = 0.0f;     // what a padding entry (source kXPad = C) looks up
        any = __syncthreads_or(any);
        const int64_t q0 = chunk_first[c] >> 2, q1 = chunk_first[c + 1] >> 2;
        const u16x4* __restrict__ sv = reinterpret_cast<const u16x4*>(x_src);
        f32x4* __restrict__ out = reinterpret_cast<f32x4*>(vals);
        // The chunk's vectors are cut into tiles of kXTile (32 KB of values); the workgroup's wavefronts
        // take the tiles in turn, so at any moment the workgroup writes a window of sixteen adjacent
        // tiles, each as a stream of 1 KB stores.  (The workgroup walking the chunk as one stream: 4.8 ms
        // per pass on the 10^8-vertex graph; a stream per wavefront, long or in tiles: 4.4 ms, the
        // rate at which this part writes long streams while it reads a third as much beside them.)
        constexpr int64_t kXTile = 2048;
        const int64_t ntile = (q1 - q0 + kXTile - 1) / kXTile;
        for (int64_t tile = threadIdx.x >> 6; tile < ntile; tile += kXBlock / kWave) {
            const int64_t wq0 = q0 + tile * kXTile;
            const int64_t wq1 = wq0 + kXTile < q1 ? wq0 + kXTile : q1;
            if (!any) {                  // nothing of this chunk is in the frontier: zeros, without reading the entries
                const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                for (int64_t q = wq0 + (threadIdx.x & (kWave - 1)); q < wq1; q += kWave) __builtin_nontemporal_store(z, out + q);
                continue;
            }
            // the next round's entries are in flight while this round's values are looked up and stored
            constexpr int64_t kRound = (int64_t)kWave * kXUnroll;
            u16x4 s[kXUnroll];
            int64_t q = wq0 + (threadIdx.x & (kWave - 1));
#pragma unroll
            for (int u = 0; u < kXUnroll; ++u)
                if (q + u * kWave < wq1) s[u] = __builtin_nontemporal_load(sv + q + u * kWave);
            for (; q < wq1; q += kRound) {
                u16x4 n[kXUnroll];
#pragma unroll
                for (int u = 0; u < kXUnroll; ++u)
                    if (q + kRound + u * kWave < wq1) n[u] = __builtin_nontemporal_load(sv + q + kRound + u * kWave);
#pragma unroll
                for (int u = 0; u < kXUnroll; ++u)
                    if (q + u * kWave < wq1) {
                        f32x4 w;
                        w.x = ych[s[u].x];
                        w.y = ych[s[u].y];
                        w.z = ych[s[u].z];
                        w.w = ych[s[u].w];
                        __builtin_nontemporal_store(w, out + q + u * kWave);
                    }
#pragma unroll
                for (int u = 0; u < kXUnroll; ++u) s[u] = n[u];
            }
        }
        __syncthreads();                 // the next chunk overwrites ych
    }
}

// Second pass.  The block's vectors form one sequence (vector q of the block: the pieces of chunks
// 0, 1, ... end to end); the j-th of `parts` equal shares of it is walked by this workgroup, a
// group of kXGroup pieces at a time: prefix[k] = first vector of piece k in that sequence, start[k]
// = where the piece lies in the arrays.  With one share per block the workgroup finishes the
// block's vertices itself (p^[h], running total, next hop's y); otherwise it leaves its sums in
// part[j] for vip_tile_finish_kernel.
__global__ void __launch_bounds__(kXBlock) vip_reduce_kernel(const float* __restrict__ vals,
                                                             const uint16_t* __restrict__ x_row,
                                                             const uint32_t* __restrict__ x_start,
                                                             const uint32_t* __restrict__ x_prefix, int nch, int parts,
                                                             int64_t N, double* __restrict__ part, int64_t part_stride,
                                                             VipHop a) {
    extern __shared__ double acc[];
    constexpr int R = 1 << kTileRowBits;
    uint32_t* prefix = reinterpret_cast<uint32_t*>(acc + R);     // [kXGroup + 1]
    uint32_t* start = prefix + kXGroup + 1;                      // [kXGroup]
    const int64_t nrb = gridDim.x / parts;
    const int64_t rb = blockIdx.x % nrb;
    const int j = (int)(blockIdx.x / nrb);
    for (int i = threadIdx.x; i < R; i += kXBlock) acc[i] = 0.0;
    const uint32_t* __restrict__ pre_b = x_prefix + rb * (nch + 1);
    const uint32_t* __restrict__ sta_b = x_start + rb * nch;
    const uint32_t nvec = pre_b[nch];
    const uint32_t beg = (uint32_t)((uint64_t)nvec * j / parts), end = (uint32_t)((uint64_t)nvec * (j + 1) / parts);
    const f32x4* __restrict__ vv = reinterpret_cast<const f32x4*>(vals);
    const u16x4* __restrict__ rv = reinterpret_cast<const u16x4*>(x_row);
    for (int g0 = 0; g0 < nch; g0 += kXGroup) {
        const int gn = nch - g0 < kXGroup ? nch - g0 : kXGroup;
        __syncthreads();                 // the tables of the group before are no longer read; acc is cleared
        for (int k = threadIdx.x; k <= gn; k += kXBlock) prefix[k] = pre_b[g0 + k];
        for (int k = threadIdx.x; k < gn; k += kXBlock) start[k] = sta_b[g0 + k];
        __syncthreads();
        const uint32_t lo = prefix[0] > beg ? prefix[0] : beg, hi = prefix[gn] < end ? prefix[gn] : end;
        if (lo >= hi) continue;          // uniform over the workgroup
        // Every wavefront takes a contiguous run of the group's vectors and walks it 64 vectors at a
        // time, so a lane's piece is found by bisection once and then moves on by a piece or two per
        // round (pieces hold some tens of vectors).  (With the workgroup striding over the group
        // together, a lane skipped some sixty pieces between two of its vectors and spent its time
        // stepping through the table: 6.6 ms per hop of the 10^8-vertex graph instead of 3.)
        const uint32_t per_wave = ((hi - lo + (kXBlock / kWave) - 1) / (kXBlock / kWave) + kWave - 1) / kWave * kWave;
        const uint32_t wlo = lo + (threadIdx.x >> 6) * per_wave;
        const uint32_t whi = wlo + per_wave < hi ? wlo + per_wave : hi;     // wlo may lie beyond hi: then nothing to do
        uint32_t q = wlo + (threadIdx.x & (kWave - 1));
        int k = 0;
        {
            int l = 0, h = gn - 1;       // last piece with prefix[k] <= q (used only where q < whi <= prefix[gn])
            while (l < h) {
                const int mid = (l + h + 1) >> 1;
                if (prefix[mid] <= q) l = mid; else h = mid - 1;
            }
            k = l;
        }
        uint32_t kend = prefix[k + 1];
        constexpr int U = 4;             // vectors in flight per lane
        f32x4 v[U];
        u16x4 r[U];
        bool ok[U];
        auto fetch = [&](int u, uint32_t qq) {
            ok[u] = qq < whi && wlo < hi;
            if (ok[u]) {
                while (qq >= kend) { ++k; kend = prefix[k + 1]; }
                const uint32_t at = start[k] + (qq - prefix[k]);
                v[u] = __builtin_nontemporal_load(vv + at);
                r[u] = __builtin_nontemporal_load(rv + at);
            }
        };
        auto add = [&](const f32x4& w, const u16x4& rr) {
            if (w.x != 0.0f) unsafeAtomicAdd(&acc[rr.x], (double)w.x);
            if (w.y != 0.0f) unsafeAtomicAdd(&acc[rr.y], (double)w.y);
            if (w.z != 0.0f) unsafeAtomicAdd(&acc[rr.z], (double)w.z);
            if (w.w != 0.0f) unsafeAtomicAdd(&acc[rr.w], (double)w.w);
        };
#pragma unroll
        for (int u = 0; u < U; ++u) fetch(u, q + u * kWave);
        while (ok[0]) {
            f32x4 cv[U];
            u16x4 cr[U];
            bool cok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) { cv[u] = v[u]; cr[u] = r[u]; cok[u] = ok[u]; }
            q += U * kWave;
            // the next round's loads are in flight while this round's sums are formed
#pragma unroll
            for (int u = 0; u < U; ++u) fetch(u, q + u * kWave);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (cok[u]) add(cv[u], cr[u]);
        }
    }
    __syncthreads();
    const int64_t u0 = rb << kTileRowBits;
    if (parts == 1) {
        unsigned long long verts = 0, edges = 0;
        for (int i = threadIdx.x; i < R; i += kXBlock)
            if (u0 + i < N) vip_finish_vertex(a, u0 + i, acc[i], verts, edges);
    } else {
        double* __restrict__ out = part + (int64_t)j * part_stride + u0;
        for (int i = threadIdx.x; i < R; i += kXBlock) out[i] = acc[i];
    }
}

// y_1(v) for the training vertices (p^[0] = min(1, B/|T|), Sec. 3.1); optionally hop 0 into the
// total; counts hop 1's frontier on the way.
__global__ void __launch_bounds__(kBlock) vip_init_kernel(const int32_t* __restrict__ T, int64_t nT, int64_t N, double p0,
                                                          double f1, const int64_t* __restrict__ rowptr,
                                                          float* __restrict__ y, double* __restrict__ tot, int include_hop0,
                                                          int* __restrict__ bad, unsigned long long* __restrict__ stat) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    unsigned long long verts = 0, edges = 0;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < nT; i += stride) {
        const int64_t v = T[i];
        if (v < 0 || v >= N) { *bad = 1; continue; }
        const int64_t d = rowptr[v + 1] - rowptr[v];
        if (d > 0) {
            double t = f1 / (double)d;
            if (t > 1.0) t = 1.0;
            const float yv = (float)log1p(-(t * p0));
            y[v] = yv;
            if (yv != 0.0f) { ++verts; edges += (unsigned long long)d; }
        }
        if (include_hop0) tot[v] = log1p(-p0);
    }
    write_frontier_stat(stat, verts, edges);
}

// ---- Proposition 1 with arbitrary initial and transition probabilities (Sec. 3.1) -------------
// Push form over the CSR, whose edge order the transition probabilities share: every vertex with
// p^[h-1](v) > 0 adds log1p(-t_h(e) p^[h-1](v)) to the fp64 sum of every member of its row.

__device__ __forceinline__ float unit_or_flag(float x, int* bad) {
    if (x >= 0.0f && x <= 1.0f) return x;
    *bad = 1;                                     // also for NaN
    return 0.0f;
}

__global__ void __launch_bounds__(kBlock) vipg_init_kernel(const float* __restrict__ p0, int64_t N,
                                                           float* __restrict__ pcur, double* __restrict__ tot,
                                                           int include_hop0, int* __restrict__ bad) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x; v < N; v += stride) {
        const float p = unit_or_flag(p0[v], bad);
        pcur[v] = p;
        if (include_hop0) tot[v] = log1p(-(double)p);
    }
}

__global__ void __launch_bounds__(kBlock) vipg_push_kernel(const int32_t* __restrict__ list,
                                                           const unsigned long long* __restrict__ nf_ptr,
                                                           const float* __restrict__ pcur,
                                                           const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ col,
                                                           const float* __restrict__ t, double* __restrict__ acc,
                                                           int* __restrict__ bad) {
    const int lane = lane_id();
    const int64_t nf = (int64_t)*nf_ptr;
    const int64_t wave = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
    for (int64_t i = wave; i < nf; i += nwaves) {
        int64_t b;
        uint32_t deg;
        const int64_t v = frontier_entry(list, i, rowptr, b, deg);
        const double pv = (double)pcur[v];
        const int64_t e = b + deg;
        for (int64_t k = b + lane; k < e; k += kWave) {
            const double x = (double)unit_or_flag(t[k], bad) * pv;
            if (x > 0.0) unsafeAtomicAdd(&acc[col[k]], log1p(-x));
        }
    }
}

// Push without global atomics, for graphs that carry the row-block structure: the fp64 global
// atomic adds of vipg_push_kernel run at about 21 G/s whatever the walk, so a dense hop of 121M
// edges takes 5.7 ms.  Here every frontier edge v -> u becomes an entry (fp32 weight, row of u
// inside its block) in the bin of u's row block, and a second kernel adds a bin's entries into the
// block's fp64 sums in LDS, as the pull over row blocks does.  A bin has room for every edge that
// ends in its block (its base and size are the block's range in the transposed structure), so no
// counting pass over the hop is needed.  A workgroup takes a portion of the frontier and lays the
// rows of its vertices end to end (prefix sums of their lengths in LDS; a wavefront takes runs of
// 64 consecutive edges of that sequence whatever the row lengths, so its loads are contiguous).
// One walk over col[] counts the portion's entries per bin in LDS, one global atomic per bin
// reserves their range (reserving per 2048 edges instead serialised on the bins' counters: 59k
// same-address atomics, 0.9 ms), and a second walk forms the entries and stores them, the slot
// inside the range coming from an LDS atomic.  (Sorting 2048 entries at a time by bin in LDS, so
// that neighbouring threads store neighbouring entries, was slower: 1.2 ms against 0.9 ms per
// dense hop; a thread taking 8 consecutive edges instead of a wavefront taking 64: 1.25 ms.)
constexpr int kBinBlock = 256;           // threads per workgroup, and most frontier vertices per portion
constexpr int kBinPer = 8;               // edges per thread and round
constexpr int kBinChunk = kBinBlock * kBinPer;
constexpr int64_t kBinMaxBlocks = 16384; // row blocks whose two counters each fit the LDS of a workgroup

// Frontier entries per portion: small frontiers are cut into small portions so that they still
// spread over the chip.
__device__ __forceinline__ int64_t bin_portion_size(int64_t nf) {
    const int64_t per = (nf + gridDim.x - 1) / gridDim.x;
    return per < kWave ? kWave : (per > kBinBlock ? kBinBlock : per);
}

// Which list entries make up a portion.  A small frontier (at most two portions per workgroup) is
// dealt out entry by entry, so that the pieces of a long row, adjacent in the list, land in
// different portions; a large one is cut into runs of consecutive entries, whose rows lie
// side by side in col[] (dealt out entry by entry, the dense hop of the general propagation took
// 1.00 ms instead of 0.88).
struct PortionMap {
    int64_t nf, per, nportions;
    bool dealt;
    __device__ __forceinline__ explicit PortionMap(int64_t nf_) : nf(nf_) {
        per = bin_portion_size(nf);
        nportions = (nf + per - 1) / per;
        dealt = nportions <= 2 * (int64_t)gridDim.x;
    }
    __device__ __forceinline__ int count(int64_t portion) const {
        if (dealt) return (int)((nf - portion + nportions - 1) / nportions);
        const int64_t rest = nf - portion * per;
        return (int)(rest < per ? rest : per);
    }
    __device__ __forceinline__ int64_t entry(int64_t portion, int t) const {
        return dealt ? portion + (int64_t)t * nportions : portion * per + t;
    }
};

struct BinPortion {
    uint32_t prefix[kBinBlock + 1];      // edges of the portion before vertex i
    int64_t  row[kBinBlock];             // where vertex i's row starts in col[] and t[]
    float    p[kBinBlock];               // p^[h-1] of vertex i
    uint32_t wave_sum[kBinBlock / kWave];
};

// Exclusive prefix sums over a workgroup of kBinBlock threads; ends with a barrier.
__device__ __forceinline__ uint32_t bin_block_scan(uint32_t v, uint32_t* wave_sum, uint32_t& total) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const uint32_t inc = (uint32_t)wave_inclusive_scan((int)v);
    if (lane == kWave - 1) wave_sum[wave] = inc;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kBinBlock / kWave; ++w) {
        const uint32_t x = wave_sum[w];
        if (w < wave) before += x;
        all += x;
    }
    total = all;
    __syncthreads();
    return before + inc - v;
}

// The vertex of the portion whose row holds edge x of the sequence (x < prefix[nv]): the last i
// with prefix[i] <= x.
__device__ __forceinline__ int bin_vertex_of(const BinPortion& po, int nv, uint32_t x) {
    int lo = 0, hi = nv;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (po.prefix[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// A thread's walk over ascending edges of the portion's sequence: where edge x sits in col[] and
// t[], and the probability of its source.  Rows are entered by comparison with the row's end, so an
// edge inside the row of the edge before costs an add.
struct BinCursor {
    int      i;          // vertex of the portion
    uint32_t row_end;    // first x beyond its row
    int64_t  shift;      // position in col[] minus x, inside this row
    float    p;
    __device__ __forceinline__ void start(const BinPortion& po, int nv, uint32_t x) {
        i = bin_vertex_of(po, nv, x);
        enter(po);
    }
    __device__ __forceinline__ void enter(const BinPortion& po) {
        row_end = po.prefix[i + 1];
        shift = po.row[i] - (int64_t)po.prefix[i];
        p = po.p[i];
    }
    __device__ __forceinline__ int64_t at(const BinPortion& po, uint32_t x) {     // x < prefix[nv], not below the x before
        if (x >= row_end) {
            do { ++i; } while (x >= po.prefix[i + 1]);
            enter(po);
        }
        return shift + (int64_t)x;
    }
};

// Edge q of a thread in the round that starts at edge c0: a wavefront takes kBinPer runs of 64
// consecutive edges, so that its loads from col[] and t[] are contiguous.
__device__ __forceinline__ uint32_t bin_edge(uint32_t c0, int q) {
    return c0 + (threadIdx.x >> 6) * (kWave * kBinPer) + (uint32_t)q * kWave + (threadIdx.x & (kWave - 1));
}

// Push form of eq. (2) for the uniform weights: every frontier vertex adds y(v) into the
// accumulator of every member of adj(v) (fp64 global atomics).  Portions of `per` frontier vertices
// walked as one edge sequence, as above: with one wavefront per vertex the longest row set the
// kernel's duration (138 us for the 1.2M out-edges of 24k training vertices, degrees up to 20k).
__global__ void __launch_bounds__(kBinBlock) vip_push_flat_kernel(const int32_t* __restrict__ list,
                                                                  const unsigned long long* __restrict__ nf_ptr,
                                                                  const float* __restrict__ y,
                                                                  const int64_t* __restrict__ rowptr,
                                                                  const int32_t* __restrict__ col,
                                                                  double* __restrict__ acc) {
    __shared__ BinPortion po;
    const int64_t nf = (int64_t)*nf_ptr;
    const PortionMap pm(nf);
    for (int64_t portion = blockIdx.x; portion < pm.nportions; portion += gridDim.x) {
        const int nv = pm.count(portion);
        const int64_t mine = pm.entry(portion, threadIdx.x);
        uint32_t deg = 0;
        if ((int)threadIdx.x < nv) {
            int64_t b;
            const int32_t v = frontier_entry(list, mine, rowptr, b, deg);
            po.row[threadIdx.x] = b;
            po.p[threadIdx.x] = y[v];
        }
        uint32_t total;
        const uint32_t ex = bin_block_scan(deg, po.wave_sum, total);
        if ((int)threadIdx.x < nv) po.prefix[threadIdx.x] = ex;
        if (threadIdx.x == 0) po.prefix[nv] = total;
        __syncthreads();
        for (uint32_t c0 = 0; c0 < total; c0 += kBinChunk) {
            if (bin_edge(c0, 0) >= total) continue;
            BinCursor cu;
            cu.start(po, nv, bin_edge(c0, 0));
            int32_t u[kBinPer];
            float w[kBinPer];
#pragma unroll
            for (int q = 0; q < kBinPer; ++q) {
                u[q] = -1;
                if (bin_edge(c0, q) < total) {
                    u[q] = col[cu.at(po, bin_edge(c0, q))];
                    w[q] = cu.p;
                }
            }
#pragma unroll
            for (int q = 0; q < kBinPer; ++q)
                if (u[q] >= 0) unsafeAtomicAdd(&acc[u[q]], (double)w[q]);       // hardware fp64 add
        }
        __syncthreads();
    }
}

// log1p(-x) for 0 < x <= 1 to a few fp32 ulp.  All terms of a vertex's sum have one sign, so the
// sum's relative error is at most the largest of its terms'; the library's fp32 and fp64 routines
// carry extended precision that is of no use here and were 90 and 117 of the walk's instructions per
// edge.  Below 1/4 the atanh series in s = x / (2 - x) <= 1/7 (six terms: the next is below 2^-33
// of the first); above, the logarithm of 1 - x, whose rounding error is at most 2^-25 against a
// result of at least 0.28.
__device__ __forceinline__ float bin_log1p_neg(float x) {
    const float s = __fdividef(x, 2.0f - x);
    const float z = s * s;
    float q = 1.0f / 11.0f;
    q = __fmaf_rn(q, z, 1.0f / 9.0f);
    q = __fmaf_rn(q, z, 1.0f / 7.0f);
    q = __fmaf_rn(q, z, 1.0f / 5.0f);
    q = __fmaf_rn(q, z, 1.0f / 3.0f);
    q = __fmaf_rn(q, z, 1.0f);
    const float small = -2.0f * s * q;
    const float large = __logf(1.0f - x);
    return x < 0.25f ? small : large;
}

__global__ void __launch_bounds__(kBinBlock) vipg_bin_fill_kernel(const int32_t* __restrict__ list,
                                                                  const unsigned long long* __restrict__ nf_ptr,
                                                                  const float* __restrict__ pcur,
                                                                  const int64_t* __restrict__ rowptr,
                                                                  const int32_t* __restrict__ col,
                                                                  const float* __restrict__ t, int rbits, int nrb,
                                                                  const int64_t* __restrict__ first, int nch,
                                                                  uint32_t* __restrict__ cursor,
                                                                  uint2* __restrict__ bins, int* __restrict__ bad) {
    __shared__ BinPortion po;
    extern __shared__ uint32_t lds_u32[];
    uint32_t* base = lds_u32;            // the portion's entries per row block, then the entry (index into bins[], below 2^32) where they start
    uint32_t* filled = lds_u32 + nrb;    // entries of the block written so far
    const int64_t nf = (int64_t)*nf_ptr;
    const PortionMap pm(nf);
    const uint32_t rmask = (1u << rbits) - 1u;
    const int bins_per_thread = (nrb + kBinBlock - 1) / kBinBlock;
    const int r0 = threadIdx.x * bins_per_thread;
    const int r1 = r0 + bins_per_thread < nrb ? r0 + bins_per_thread : nrb;
    // Portions are handed out through a counter (the slot after the bins' cursors): their sizes
    // differ by the degrees of their vertices, and with fixed shares half of the wavefronts had
    // left before the kernel's end.
    __shared__ uint32_t portion;
    for (;;) {
        if (threadIdx.x == 0) portion = atomicAdd(&cursor[nrb], 1u);
        __syncthreads();
        if ((int64_t)portion >= pm.nportions) break;
        const int nv = pm.count(portion);
        const int64_t mine = pm.entry(portion, threadIdx.x);
        uint32_t deg = 0;
        if ((int)threadIdx.x < nv) {
            int64_t b;
            const int32_t v = frontier_entry(list, mine, rowptr, b, deg);
            po.row[threadIdx.x] = b;
            po.p[threadIdx.x] = pcur[v];
        }
        uint32_t total;
        const uint32_t ex = bin_block_scan(deg, po.wave_sum, total);
        if ((int)threadIdx.x < nv) po.prefix[threadIdx.x] = ex;
        if (threadIdx.x == 0) po.prefix[nv] = total;
        for (int r = threadIdx.x; r < nrb; r += kBinBlock) base[r] = 0u;
        __syncthreads();                                   // publishes prefix[], row[], p[]
        // first walk: the portion's entries per bin
        for (uint32_t c0 = 0; c0 < total; c0 += kBinChunk) {
            if (bin_edge(c0, 0) >= total) continue;
            BinCursor cu;
            cu.start(po, nv, bin_edge(c0, 0));
            uint32_t u[kBinPer];
#pragma unroll
            for (int q = 0; q < kBinPer; ++q) u[q] = bin_edge(c0, q) < total ? (uint32_t)col[cu.at(po, bin_edge(c0, q))] : ~0u;
#pragma unroll
            for (int q = 0; q < kBinPer; ++q)
                if (u[q] != ~0u) atomicAdd(&base[u[q] >> rbits], 1u);
        }
        __syncthreads();
        for (int r = r0; r < r1; ++r) {
            const uint32_t c = base[r];
            base[r] = (uint32_t)first[(int64_t)r * nch] + (c ? atomicAdd(&cursor[r], c) : 0u);
            filled[r] = 0u;
        }
        __syncthreads();
        // second walk: the entries
        for (uint32_t c0 = 0; c0 < total; c0 += kBinChunk) {
            if (bin_edge(c0, 0) >= total) continue;
            BinCursor cu;
            cu.start(po, nv, bin_edge(c0, 0));
            uint32_t key[kBinPer];
            float pv[kBinPer], tv[kBinPer];
#pragma unroll
            for (int q = 0; q < kBinPer; ++q) {
                key[q] = ~0u;
                if (bin_edge(c0, q) < total) {
                    const int64_t k = cu.at(po, bin_edge(c0, q));
                    key[q] = (uint32_t)col[k];
                    tv[q] = t[k];
                    pv[q] = cu.p;
                }
            }
#pragma unroll
            for (int q = 0; q < kBinPer; ++q) {
                if (key[q] != ~0u) {
                    const uint32_t u = key[q];
                    const float xw = unit_or_flag(tv[q], bad) * pv[q];
                    const uint32_t rb = u >> rbits;
                    const uint32_t slot = atomicAdd(&filled[rb], 1u);
                    bins[base[rb] + slot] = make_uint2(__float_as_uint(xw > 0.0f ? bin_log1p_neg(xw) : 0.0f), u & rmask);
                }
            }
        }
        __syncthreads();
    }
}

// Adds the entries of one share of one bin into the block's fp64 sums (LDS) and writes them to
// part[j][row], like vip_tile_kernel but with the weights already in place.
__global__ void __launch_bounds__(kTileBlock) vip_bin_sum_kernel(const uint2* __restrict__ bins,
                                                                 const uint32_t* __restrict__ cursor,
                                                                 const int64_t* __restrict__ first, int nch, int parts,
                                                                 int rbits, double* __restrict__ part, int64_t part_stride) {
    extern __shared__ double acc[];
    const int R = 1 << rbits;
    const int64_t rb = blockIdx.x / parts;
    const int j = blockIdx.x % parts;
    for (int i = threadIdx.x; i < R; i += kTileBlock) acc[i] = 0.0;
    __syncthreads();
    const int64_t b0 = first[rb * nch], len = (int64_t)cursor[rb];
    const int64_t beg = b0 + len * j / parts, end = b0 + len * (j + 1) / parts;
    for (int64_t e = beg + threadIdx.x; e < end; e += kTileBlock) {
        const unsigned long long x = __builtin_nontemporal_load(reinterpret_cast<const unsigned long long*>(bins) + e);
        const uint32_t w = (uint32_t)x;                    // .x of the entry
        if (w != 0u) unsafeAtomicAdd(&acc[(uint32_t)(x >> 32)], (double)__uint_as_float(w));
    }
    __syncthreads();
    double* __restrict__ out = part + (int64_t)j * part_stride + (rb << rbits);
    for (int i = threadIdx.x; i < R; i += kTileBlock) out[i] = acc[i];
}

__global__ void __launch_bounds__(kBlock) vipg_finish_kernel(const double* __restrict__ acc, double* __restrict__ tot,
                                                             int first, int last, float* __restrict__ p_hop,
                                                             float* __restrict__ p_total, float* __restrict__ pnext,
                                                             int64_t N, int parts, int64_t part_stride) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x; u < N; u += stride) {
        double S = acc[u];
        for (int j = 1; j < parts; ++j) S += acc[(int64_t)j * part_stride + u];
        const double ph = -expm1(S);
        if (p_hop) p_hop[u] = (float)ph;
        const double T = first ? S : tot[u] + S;
        if (last) p_total[u] = (float)(-expm1(T));
        else { tot[u] = T; pnext[u] = (float)ph; }
    }
}

}  // namespace spp

extern "C" int spp_vip_propagate_general(spp_ctx* ctx, const spp_graph* g, const float* d_p0,
                                         const float* const* d_t, int32_t L, float* d_p_total, float* d_p_hop,
                                         uint32_t flags) {
    using namespace spp;
    SPP_CHECK(ctx && g && d_p0 && d_t && d_p_total, SPP_E_ARG, "spp_vip_propagate_general: null argument");
    SPP_CHECK(L >= 1 && L <= SPP_MAX_L, SPP_E_ARG, "spp_vip_propagate_general: L = %d not in [1, %d]", L, SPP_MAX_L);
    for (int h = 0; h < L; ++h)
        SPP_CHECK(d_t[h] || g->M == 0, SPP_E_ARG, "spp_vip_propagate_general: no transition probabilities for hop %d", h + 1);
    SPP_HIP(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;
    const int64_t N = g->N;
    SPP_TRY(ctx->y0.reserve((size_t)N * sizeof(float)));
    SPP_TRY(ctx->y1.reserve((size_t)N * sizeof(float)));
    SPP_TRY(ctx->tot.reserve((size_t)N * sizeof(double) + sizeof(int)));
    SPP_TRY(ctx->acc.reserve((size_t)N * sizeof(double)));
    const int64_t lcap = frontier_list_capacity(N, g->M);
    SPP_TRY(ctx->frontier.reserve((size_t)(lcap + 2) * sizeof(int32_t) + 4 * sizeof(unsigned long long)));
    int32_t* flist = ctx->frontier.as<int32_t>();
    unsigned long long* fcount = reinterpret_cast<unsigned long long*>(flist + (lcap + (lcap & 1)));
    float* pcur = ctx->y0.as<float>();
    float* pnext = ctx->y1.as<float>();
    double* tot = ctx->tot.as<double>();
    double* acc = ctx->acc.as<double>();
    int* d_bad = reinterpret_cast<int*>(tot + N);
    const int include0 = (flags & SPP_VIP_INCLUDE_HOP0) ? 1 : 0;
    const int fill_grid = ctx->num_cu * 8;
    // With the row-block structure at hand the push goes through bins (no global fp64 atomics).
    const bool binned = g->has_in && g->nrb > 0 && g->nrb <= kBinMaxBlocks && g->M > 0;
    int parts = 1;
    const int64_t part_stride = binned ? g->nrb << g->tile_rbits : N;
    uint2* bins = nullptr;
    uint32_t* cursor = nullptr;
    const size_t fill_lds = binned ? 2 * (size_t)g->nrb * sizeof(uint32_t) : 0;
    const size_t sum_lds = binned ? sizeof(double) << g->tile_rbits : 0;
    if (binned) {
        const int64_t want = ((int64_t)ctx->num_cu * 4 + g->nrb - 1) / g->nrb;
        parts = (int)(want < 1 ? 1 : (want > 16 ? 16 : want));
        SPP_TRY(ctx->acc.reserve((size_t)parts * (size_t)part_stride * sizeof(double)));
        acc = ctx->acc.as<double>();
        SPP_TRY(ctx->bins.reserve(((size_t)g->M + (size_t)g->nrb + 1) * sizeof(uint2)));
        bins = ctx->bins.as<uint2>();
        cursor = reinterpret_cast<uint32_t*>(bins + g->M);
        if (ctx->bin_lds_set < (int)fill_lds) {
            SPP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&vipg_bin_fill_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)fill_lds));
            ctx->bin_lds_set = (int)fill_lds;
        }
        if (ctx->sum_lds_set < (int)sum_lds) {
            SPP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&vip_bin_sum_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)sum_lds));
            ctx->sum_lds_set = (int)sum_lds;
        }
    }
    {
        ScopedTimer tt(ctx, SPP_T_VIP_TOTAL, st);
        fill_f32_kernel<<<1, 64, 0, st>>>(reinterpret_cast<float*>(d_bad), 1, 0.f);
        vipg_init_kernel<<<fill_grid, kBlock, 0, st>>>(d_p0, N, pcur, tot, include0, d_bad);
        for (int h = 1; h <= L; ++h) {
            ScopedTimer th(ctx, SPP_T_VIP_HOP_FIRST + h - 1, st);
            fill_f64_kernel<<<1, 64, 0, st>>>(reinterpret_cast<double*>(fcount), 3, 0.0);
            launch_frontier_list(fill_grid, st, pcur, g->rowptr, N, flist, fcount + 2);
            if (binned) {
                fill_f32_kernel<<<(unsigned)((g->nrb + kBlock) / kBlock), kBlock, 0, st>>>(
                    reinterpret_cast<float*>(cursor), g->nrb + 1, 0.f);         // all-zero bits either way
                // a bin is the range of the edges that end in its row block: block_first, with a stride of one
                vipg_bin_fill_kernel<<<ctx->num_cu * 8, kBinBlock, fill_lds, st>>>(
                    flist, fcount + 2, pcur, g->rowptr, g->col, d_t[h - 1], g->tile_rbits, (int)g->nrb,
                    g->block_first, 1, cursor, bins, d_bad);
                vip_bin_sum_kernel<<<(unsigned)(g->nrb * parts), kTileBlock, sum_lds, st>>>(
                    bins, cursor, g->block_first, 1, parts, g->tile_rbits, acc, part_stride);
            } else {
                fill_f64_kernel<<<fill_grid, kBlock, 0, st>>>(acc, N, 0.0);
                vipg_push_kernel<<<ctx->num_cu * 32, kBlock, 0, st>>>(flist, fcount + 2, pcur, g->rowptr, g->col,
                                                                     d_t[h - 1], acc, d_bad);
            }
            vipg_finish_kernel<<<fill_grid, kBlock, 0, st>>>(acc, tot, (h == 1 && !include0) ? 1 : 0, h == L ? 1 : 0,
                                                             d_p_hop ? d_p_hop + (int64_t)(h - 1) * N : nullptr,
                                                             d_p_total, pnext, N, parts, part_stride);
            ctx->vip_pushed[h - 1] = 1;
            ctx->vip_frontier_edges[h - 1] = -1;
            float* tmp = pcur; pcur = pnext; pnext = tmp;
        }
    }
    SPP_HIP(hipGetLastError());
    if (flags & SPP_SYNC) {
        int bad = 0;
        SPP_HIP(hipMemcpyAsync(&bad, d_bad, sizeof(int), hipMemcpyDeviceToHost, st));
        SPP_HIP(hipStreamSynchronize(st));
        SPP_CHECK(bad == 0, SPP_E_ARG, "spp_vip_propagate_general: a probability lies outside [0, 1]; it was taken as 0");
    }
    return SPP_OK;
}

extern "C" int spp_vip_propagate(spp_ctx* ctx, const spp_graph* g, const int32_t* d_T, int64_t nT,
                                 int32_t B, const int32_t* fanouts, int32_t L,
                                 float* d_p_total, float* d_p_hop, uint32_t flags) {
    using namespace spp;
    SPP_CHECK(ctx && g && d_T && fanouts && d_p_total, SPP_E_ARG, "spp_vip_propagate: null argument");
    SPP_CHECK(g->has_in, SPP_E_ARG, "spp_vip_propagate: the graph was created without SPP_GRAPH_IN_LISTS");
    SPP_CHECK(L >= 1 && L <= SPP_MAX_L, SPP_E_ARG, "spp_vip_propagate: L = %d not in [1, %d]", L, SPP_MAX_L);
    SPP_CHECK(nT > 0 && B > 0, SPP_E_ARG, "spp_vip_propagate: nT = %lld, B = %d must be positive", (long long)nT, B);
    for (int h = 0; h < L; ++h)
        SPP_CHECK(fanouts[h] >= 1, SPP_E_ARG, "spp_vip_propagate: fanout %d of hop %d", fanouts[h], h + 1);
    SPP_HIP(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;
    const int64_t N = g->N;
    SPP_TRY(ctx->y0.reserve((size_t)N * sizeof(float)));
    SPP_TRY(ctx->y1.reserve((size_t)N * sizeof(float)));
    SPP_TRY(ctx->tot.reserve((size_t)N * sizeof(double) + sizeof(int)));
    // dense hops over row blocks: shares per block for at most four workgroups per CU (on 147 blocks
    // and 256 CUs, in block-major order: 6 shares 224 + 31 us for the kernel and the finish, 7 shares 234 + 34,
    // 8 shares 279 + 38; in share-major order 6 shares 214 + 31, 8 shares 209 + 37)
    int parts = 1;
    if (g->nrb > 0) {
        const int64_t want = (int64_t)ctx->num_cu * 4 / g->nrb;
        parts = (int)(want < 1 ? 1 : (want > 16 ? 16 : want));
    }
    // the chunked layout: with a row block per CU or more, one workgroup takes a whole block and
    // finishes its vertices itself (no partial sums leave the chip)
    if (g->has_x && g->nrb >= ctx->num_cu) parts = 1;
    const int64_t part_stride = g->nrb << g->tile_rbits;
    {
        const size_t tile_bytes = (size_t)parts * (size_t)part_stride * sizeof(double);
        const size_t push_bytes = (size_t)N * sizeof(double);
        SPP_TRY(ctx->acc.reserve(tile_bytes > push_bytes ? tile_bytes : push_bytes));
    }
    const size_t lds_bytes = (sizeof(double) << g->tile_rbits) + (size_t)(g->nch + 1) * sizeof(uint32_t);
    const size_t x_lds_expand = (sizeof(float) << kXSrcBits) + sizeof(float);
    static_assert(kXPad == (1u << kXSrcBits), "a padding entry indexes the slot after the chunk's values");
    const size_t x_lds_reduce = (sizeof(double) << kTileRowBits) + (2 * kXGroup + 1) * sizeof(uint32_t);
    if (!g->has_x && ctx->tile_lds_set < (int)lds_bytes) {        // more than the 64 KB a launch may ask for by default
        SPP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&vip_tile_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
        ctx->tile_lds_set = (int)lds_bytes;
    }
    if (g->has_x) {
        if (!ctx->x_lds_set) {
            SPP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&vip_expand_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)x_lds_expand));
            SPP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&vip_reduce_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)x_lds_reduce));
            ctx->x_lds_set = 1;
        }
        SPP_TRY(ctx->xvals.reserve((size_t)(g->x_entries > 0 ? g->x_entries : 4) * sizeof(float)));
    }
    // the kernels that write a hop's y run this many workgroups; each leaves the size of the part of
    // the next frontier it saw (at most kStatBlocks pairs fit the pinned mirror)
    const int fill_grid = ctx->num_cu * 8 < kStatBlocks ? ctx->num_cu * 8 : kStatBlocks;
    const int64_t lcap = frontier_list_capacity(N, g->M);
    SPP_TRY(ctx->frontier.reserve((size_t)(lcap + 2) * sizeof(int32_t) + (4 + 2 * (size_t)kStatBlocks) * sizeof(unsigned long long)));
    int32_t* flist = ctx->frontier.as<int32_t>();
    unsigned long long* fcount = reinterpret_cast<unsigned long long*>(flist + (lcap + (lcap & 1)));    // [2]: cursor of the list
    unsigned long long* fstat = fcount + 4;
    float* ycur = ctx->y0.as<float>();
    float* ynext = ctx->y1.as<float>();
    double* tot = ctx->tot.as<double>();
    int* d_bad = reinterpret_cast<int*>(tot + N);
    const int include0 = (flags & SPP_VIP_INCLUDE_HOP0) ? 1 : 0;
    double p0 = (double)B / (double)nT;
    if (p0 > 1.0) p0 = 1.0;

    {
        ScopedTimer tt(ctx, SPP_T_VIP_TOTAL, st);
        fill_f32_kernel<<<fill_grid, kBlock, 0, st>>>(ycur, N, 0.f);
        if (include0) fill_f64_kernel<<<fill_grid, kBlock, 0, st>>>(tot, N, 0.0);
        fill_f32_kernel<<<1, 64, 0, st>>>(reinterpret_cast<float*>(d_bad), 1, 0.f);
        vip_init_kernel<<<fill_grid, kBlock, 0, st>>>(d_T, nT, N, p0, (double)fanouts[0], g->rowptr, ycur, tot, include0,
                                                      d_bad, fstat);
        bool prev_pulled = false;
        for (int h = 1; h <= L; ++h) {
            ScopedTimer th(ctx, SPP_T_VIP_HOP_FIRST + h - 1, st);
            VipHop a;
            a.rowptr = g->rowptr;
            a.y = ycur; a.y_next = ynext; a.tot = tot;
            a.p_hop = d_p_hop ? d_p_hop + (int64_t)(h - 1) * N : nullptr;
            a.p_total = d_p_total;
            a.f_next = h < L ? (double)fanouts[h] : 0.0;
            a.first = (h == 1 && !include0) ? 1 : 0;
            a.last = (h == L) ? 1 : 0;
            a.stat = fstat;
            // frontier of this hop and its out-edges, as counted by the kernel that wrote this hop's y;
            // a small frontier is pushed, a large one pulled
            // (after a pulled hop the next one is pulled without asking: frontiers that have grown large
            // rarely shrink, either form is correct for any frontier, and the question costs a host
            // round trip of about 25 us)
            unsigned long long fc[2] = {0, 0};
            if (!prev_pulled) {
                const unsigned long long* hs = reinterpret_cast<const unsigned long long*>(ctx->h_pinned + kStatMirror);
                SPP_HIP(hipMemcpyAsync(ctx->h_pinned + kStatMirror, fstat, 2 * (size_t)fill_grid * sizeof(unsigned long long),
                                       hipMemcpyDeviceToHost, st));
                SPP_HIP(hipStreamSynchronize(st));
                for (int b = 0; b < fill_grid; ++b) { fc[0] += hs[2 * b]; fc[1] += hs[2 * b + 1]; }
            }
            const bool push = !prev_pulled && (int64_t)fc[1] * kPushShare <= g->M;
            if (push) {
                double* acc = ctx->acc.as<double>();
                fill_f64_kernel<<<fill_grid, kBlock, 0, st>>>(acc, N, 0.0);
                if (fc[0] > 0) {
                    fill_f64_kernel<<<1, 64, 0, st>>>(reinterpret_cast<double*>(fcount + 2), 1, 0.0);
                    launch_frontier_list(fill_grid, st, ycur, g->rowptr, N, flist, fcount + 2);
                    // at most this many list entries (vertices and pieces of long rows); the kernel reads the count itself
                    const int64_t entries = (int64_t)fc[0] + (int64_t)fc[1] / kPieceEdges;
                    const int64_t pgrid = (int64_t)ctx->num_cu * 8, need = (entries + kWave - 1) / kWave;
                    vip_push_flat_kernel<<<(unsigned)(need < pgrid ? need : pgrid), kBinBlock, 0, st>>>(
                        flist, fcount + 2, ycur, g->rowptr, g->col, acc);
                }
                vip_push_finish_kernel<<<fill_grid, kBlock, 0, st>>>(a, acc, N);
            } else if (g->has_x) {
                const int egrid = g->x_nch < ctx->num_cu * 4 ? g->x_nch : ctx->num_cu * 4;
                vip_expand_kernel<<<egrid, kXBlock, x_lds_expand, st>>>(g->x_src, g->x_chunk_first, g->x_nch, N, ycur,
                                                                        ctx->xvals.as<float>());
                vip_reduce_kernel<<<(unsigned)(g->nrb * parts), kXBlock, x_lds_reduce, st>>>(
                    ctx->xvals.as<float>(), g->x_row, g->x_start, g->x_prefix, g->x_nch, parts, N, ctx->acc.as<double>(),
                    part_stride, a);
                if (parts > 1) vip_tile_finish_kernel<<<fill_grid, kBlock, 0, st>>>(a, ctx->acc.as<double>(), parts, part_stride, N);
            } else {
                vip_tile_kernel<<<(unsigned)(g->nrb * parts), kTileBlock, lds_bytes, st>>>(
                    g->t_edge, g->tile_first, g->nch, parts, g->tile_rbits, ycur, ctx->acc.as<double>(), part_stride);
                vip_tile_finish_kernel<<<fill_grid, kBlock, 0, st>>>(a, ctx->acc.as<double>(), parts, part_stride, N);
            }
            ctx->vip_pushed[h - 1] = push ? 1 : 0;
            ctx->vip_frontier_edges[h - 1] = prev_pulled ? -1 : (int64_t)fc[1];     // -1: not asked
            prev_pulled = !push;
            float* t = ycur; ycur = ynext; ynext = t;
        }
    }
    SPP_HIP(hipGetLastError());
    // training ids are checked on the device; the flag is read when the caller asks to wait
    if (flags & SPP_SYNC) {
        int bad = 0;
        SPP_HIP(hipMemcpyAsync(&bad, d_bad, sizeof(int), hipMemcpyDeviceToHost, st));
        SPP_HIP(hipStreamSynchronize(st));
        SPP_CHECK(bad == 0, SPP_E_ARG, "spp_vip_propagate: a training vertex id lies outside [0, N)");
    }
    return SPP_OK;
}
