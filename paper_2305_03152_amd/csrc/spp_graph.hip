// Graph handle: wraps the caller's CSR and, on request, builds the transposed structure that the
// pull form of Proposition 1, eq. (2), walks, in one of two layouts.
//   Row blocks (graphs up to 2^23 vertices, whose per-vertex vector y stays in the caches): the edges
//   v -> u grouped by blocks of 2^14 destination rows u and, inside a block, sorted by source v,
//   4 bytes per edge (the low 18 bits of the source and the row inside the block; a table says where
//   each run of 2^18 sources starts in each block).
//   Chunked (larger graphs): the edges sorted by (chunk of 2^15 sources, row block, source), every
//   (chunk, row block) piece padded to a multiple of four entries, 2 + 2 bytes per entry (source
//   inside the chunk, row inside the block), with tables for both walks: where every chunk starts,
//   and per row block where each chunk's piece lies and how many vectors precede it.
// Either is built once per graph by a radix sort of packed edge keys, then read back and compared
// with the edges it was built from before anything walks it.
#include "spp_common.h"
#include "spp_device.h"

#include <new>

namespace spp {

// Every kernel of the library indexes with these arrays, so they are checked once here: offsets
// monotone inside [0, M], column ids inside [0, N).
__global__ void __launch_bounds__(kBlock) validate_csr_kernel(int64_t N, int64_t M, const int64_t* __restrict__ rowptr,
                                                              const int32_t* __restrict__ col, int* __restrict__ bad) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    for (int64_t v = t; v < N; v += stride) {
        const int64_t b = rowptr[v], e = rowptr[v + 1];
        if (b < 0 || e > M || b > e) *bad = 1;
    }
    for (int64_t i = t; i < M; i += stride) {
        const int32_t u = col[i];
        if (u < 0 || u >= N) *bad = 1;
    }
}

__global__ void fill_i64_kernel(int64_t* p, int64_t n, int64_t v) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

// key[e] = (row block of u, v, u inside its block) for the e-th edge v -> u of the CSR.
__global__ void __launch_bounds__(kBlock) tile_keys_kernel(int64_t N, const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ col, int rbits, int vbits,
                                                           uint64_t* __restrict__ keys) {
    const int lane = lane_id();
    const int64_t wave = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
    const uint64_t rmask = (1ull << rbits) - 1;
    for (int64_t v = wave; v < N; v += nwaves) {
        const int64_t b = rowptr[v], e = rowptr[v + 1];
        for (int64_t i = b + lane; i < e; i += kWave) {
            const uint64_t u = (uint64_t)(uint32_t)col[i];          // validated at graph creation
            keys[i] = ((u >> rbits) << (vbits + rbits)) | ((uint64_t)v << rbits) | (u & rmask);
        }
    }
}

// From the sorted keys: the edge words, and first[g] = first e whose (row block, source chunk)
// index g = block * nch + chunk is >= g (indices after the last one keep the value M they were
// filled with).
__global__ void __launch_bounds__(kBlock) tile_lists_kernel(const uint64_t* __restrict__ keys, int64_t M, int rbits,
                                                            int vbits, int nch, uint32_t* __restrict__ t_edge,
                                                            int64_t* __restrict__ first) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const uint64_t rmask = (1ull << rbits) - 1, vmask = (1ull << vbits) - 1;
    auto index_of = [&](uint64_t k) {
        return (int64_t)(k >> (vbits + rbits)) * nch + (int64_t)(((k >> rbits) & vmask) >> kTileSrcLoBits);
    };
    for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < M; e += stride) {
        const uint64_t k = keys[e];
        const uint32_t v = (uint32_t)((k >> rbits) & vmask);
        t_edge[e] = ((v & ((1u << kTileSrcLoBits) - 1u)) << kTileRowBits) | (uint32_t)(k & rmask);
        const int64_t g = index_of(k);
        const int64_t prev = e > 0 ? index_of(keys[e - 1]) : -1;
        for (int64_t r = prev + 1; r <= g; ++r) first[r] = e;
    }
}

// Reads the structure back the way the propagation kernel does and compares every edge with the
// sorted key it was made from, so that a kernel that gathers through it never sees a source or a
// row out of range.  One workgroup per row block; the block's chunk bounds sit in LDS.
__global__ void __launch_bounds__(kBlock) tile_verify_kernel(const uint64_t* __restrict__ keys, int rbits, int vbits,
                                                             int nch, const uint32_t* __restrict__ t_edge,
                                                             const int64_t* __restrict__ first, int64_t N, int64_t M,
                                                             int* __restrict__ bad) {
    extern __shared__ uint32_t bound[];
    const uint64_t rmask = (1ull << rbits) - 1, vmask = (1ull << vbits) - 1;
    for (int64_t rb = blockIdx.x; rb * ((int64_t)1 << rbits) < N; rb += gridDim.x) {
        const int64_t b0 = first[rb * nch], len = first[(rb + 1) * nch] - b0;
        if (b0 < 0 || len < 0 || b0 + len > M || len > 0xFFFFFFFFll) { if (threadIdx.x == 0) *bad = 1; continue; }
        __syncthreads();
        for (int c = threadIdx.x; c <= nch; c += kBlock) bound[c] = (uint32_t)(first[rb * nch + c] - b0);
        __syncthreads();
        for (int64_t p = threadIdx.x; p < len; p += kBlock) {
            const uint64_t k = keys[b0 + p];
            const uint32_t w = t_edge[b0 + p];
            const int c = tile_chunk_of(bound, nch, (uint32_t)p);
            const bool ok = (int64_t)(k >> (vbits + rbits)) == rb && tile_source(w, c) == (uint32_t)((k >> rbits) & vmask) &&
                            (w & kTileRowMask) == (uint32_t)(k & rmask) && (int64_t)tile_source(w, c) < N &&
                            (rb << rbits) + (int64_t)(w & kTileRowMask) < N;
            if (!ok) *bad = 1;
        }
    }
}

__global__ void block_first_from_tiles_kernel(const int64_t* __restrict__ tile_first, int nch, int64_t nrb,
                                              int64_t* __restrict__ block_first) {
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b <= nrb) block_first[b] = tile_first[b * nch];
}

// The edges grouped by destination row block and sorted by source inside a block.
static int build_tiles(spp_ctx* ctx, spp_graph* g) {
    hipStream_t st = ctx->stream;
    const int64_t N = g->N, M = g->M;
    const int grid = ctx->num_cu * 8;
    int lds = 0;
    SPP_HIP(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, ctx->device));
    const int nch = (int)((N + ((int64_t)1 << kTileSrcLoBits) - 1) >> kTileSrcLoBits);
    // the fp64 sums of a block and the block's chunk bounds share the LDS of a workgroup
    const size_t bound_bytes = (size_t)(nch + 1) * sizeof(uint32_t);
    const int rbits = (size_t)lds >= (sizeof(double) << kTileRowBits) + bound_bytes + 1024 ? kTileRowBits : kTileRowBits - 1;
    SPP_CHECK((size_t)lds >= (sizeof(double) << rbits) + bound_bytes + 1024, SPP_E_HIP,
              "row blocks: %d bytes of LDS per workgroup do not hold a block's sums and chunk bounds", lds);
    int vbits = 1;
    while (((int64_t)1 << vbits) < N) ++vbits;
    const int64_t nrb = (N + ((int64_t)1 << rbits) - 1) >> rbits;
    int bbits = 1;
    while (((int64_t)1 << bbits) < nrb) ++bbits;
    g->tile_rbits = rbits; g->nrb = nrb; g->nch = nch;
    const int64_t nfirst = nrb * nch + 1;
    SPP_HIP(hipMalloc(&g->tile_first, (size_t)nfirst * sizeof(int64_t)));
    SPP_HIP(hipMalloc(&g->t_edge, (size_t)(M > 0 ? M : 1) * sizeof(uint32_t)));
    fill_i64_kernel<<<grid, kBlock, 0, st>>>(g->tile_first, nfirst, M);
    if (M > 0) {
        uint64_t *ka = nullptr, *kb = nullptr, *sorted = nullptr;
        int* d_bad = nullptr;
        SPP_HIP(hipMalloc(&ka, (size_t)M * sizeof(uint64_t)));
        hipError_t e = hipMalloc(&kb, (size_t)M * sizeof(uint64_t));
        if (e == hipSuccess) e = hipMalloc(&d_bad, sizeof(int));
        if (e != hipSuccess) {
            (void)hipFree(ka); if (kb) (void)hipFree(kb);
            set_error("row blocks: out of device memory for sort keys");
            return SPP_E_OOM;
        }
        tile_keys_kernel<<<grid, kBlock, 0, st>>>(N, g->rowptr, g->col, rbits, vbits, ka);
        int rc = radix_sort_u64(ctx, ka, kb, M, rbits, rbits + vbits + bbits, &sorted);
        if (rc == SPP_OK) {
            int bad = 0;
            tile_lists_kernel<<<grid, kBlock, 0, st>>>(sorted, M, rbits, vbits, nch, g->t_edge, g->tile_first);
            hipError_t e2 = hipMemsetAsync(d_bad, 0, sizeof(int), st);
            if (e2 == hipSuccess) {
                const int vgrid = (int)(nrb < (int64_t)ctx->num_cu * 8 ? nrb : (int64_t)ctx->num_cu * 8);
                tile_verify_kernel<<<vgrid, kBlock, bound_bytes, st>>>(sorted, rbits, vbits, nch, g->t_edge, g->tile_first,
                                                                       N, M, d_bad);
                e2 = hipMemcpyAsync(&bad, d_bad, sizeof(int), hipMemcpyDeviceToHost, st);
            }
            if (e2 == hipSuccess) e2 = hipStreamSynchronize(st);
            if (e2 != hipSuccess) { set_error("row blocks: %s", hipGetErrorString(e2)); rc = SPP_E_HIP; }
            else if (bad) { set_error("row blocks: the structure does not read back as the edges it was built from"); rc = SPP_E_HIP; }
        }
        (void)hipFree(ka); (void)hipFree(kb); (void)hipFree(d_bad);
        SPP_TRY(rc);
    }
    SPP_HIP(hipMalloc(&g->block_first, (size_t)(nrb + 1) * sizeof(int64_t)));
    block_first_from_tiles_kernel<<<(unsigned)((nrb + 1 + kBlock - 1) / kBlock), kBlock, 0, st>>>(g->tile_first, nch, nrb, g->block_first);
    SPP_HIP(hipStreamSynchronize(st));
    return SPP_OK;
}


// ---- the chunked layout ------------------------------------------------------------------------
// key[e] = (source chunk, row block, source inside the chunk, row inside the block) for the e-th
// edge v -> u of the CSR.
__global__ void __launch_bounds__(kBlock) x_keys_kernel(int64_t N, const int64_t* __restrict__ rowptr,
                                                        const int32_t* __restrict__ col, int bbits,
                                                        uint64_t* __restrict__ keys) {
    const int lane = lane_id();
    const int64_t wave = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * kBlock) >> 6;
    constexpr int lo_bits = kXSrcBits + kTileRowBits;
    for (int64_t v = wave; v < N; v += nwaves) {
        const int64_t b = rowptr[v], e = rowptr[v + 1];
        const uint64_t vc = (uint64_t)v >> kXSrcBits, vl = (uint64_t)v & ((1u << kXSrcBits) - 1u);
        for (int64_t i = b + lane; i < e; i += kWave) {
            const uint64_t u = (uint64_t)(uint32_t)col[i];          // validated at graph creation
            keys[i] = (vc << (lo_bits + bbits)) | ((u >> kTileRowBits) << lo_bits) | (vl << kTileRowBits) | (u & kTileRowMask);
        }
    }
}

// Piece index (chunk-major) of a key.
__device__ __forceinline__ int64_t x_piece_of(uint64_t k, int bbits, int64_t nrb) {
    constexpr int lo_bits = kXSrcBits + kTileRowBits;
    return (int64_t)(k >> (lo_bits + bbits)) * nrb + (int64_t)((k >> lo_bits) & ((1ull << bbits) - 1));
}

// first[g] = first sorted edge whose piece index is >= g (entries beyond the last piece keep the M
// they were filled with).
__global__ void __launch_bounds__(kBlock) x_bounds_kernel(const uint64_t* __restrict__ keys, int64_t M, int bbits,
                                                          int64_t nrb, int64_t* __restrict__ first) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < M; e += stride) {
        const int64_t g = x_piece_of(keys[e], bbits, nrb);
        const int64_t prev = e > 0 ? x_piece_of(keys[e - 1], bbits, nrb) : -1;
        for (int64_t r = prev + 1; r <= g; ++r) first[r] = e;
    }
}

// Exclusive prefix sums of the padded piece sizes, in three steps: per 1024 pieces a sum, the sums
// scanned by one workgroup, then the pieces' own offsets.  padded[npieces] = all entries.
constexpr int kXScanPer = 4;
__device__ __forceinline__ int64_t x_padded_len(const int64_t* first, int64_t g) {
    return (first[g + 1] - first[g] + 3) & ~(int64_t)3;
}
__global__ void __launch_bounds__(kBlock) x_scan_sums_kernel(const int64_t* __restrict__ first, int64_t npieces,
                                                             int64_t* __restrict__ sums) {
    __shared__ long long red[kBlock / kWave];
    const int64_t g0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * kXScanPer;
    long long acc = 0;
    for (int k = 0; k < kXScanPer; ++k)
        if (g0 + k < npieces) acc += x_padded_len(first, g0 + k);
    for (int off = kWave / 2; off > 0; off >>= 1) acc += __shfl_down(acc, off, kWave);
    if (lane_id() == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) sums[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}
__global__ void __launch_bounds__(kBlock) x_scan_top_kernel(int64_t* __restrict__ sums, int64_t n) {
    __shared__ long long wsum[kBlock / kWave];
    __shared__ long long carry_lds;
    if (threadIdx.x == 0) carry_lds = 0;
    __syncthreads();
    for (int64_t base = 0; base < n; base += kBlock) {
        const int64_t i = base + threadIdx.x;
        const long long v = i < n ? sums[i] : 0;
        long long inc = v;
        const int lane = lane_id(), wave = threadIdx.x >> 6;
        for (int off = 1; off < kWave; off <<= 1) {
            const long long t = __shfl_up(inc, off, kWave);
            if (lane >= off) inc += t;
        }
        if (lane == kWave - 1) wsum[wave] = inc;
        __syncthreads();
        long long before = carry_lds;
        for (int w = 0; w < wave; ++w) before += wsum[w];
        if (i < n) sums[i] = before + inc - v;
        __syncthreads();
        if (threadIdx.x == kBlock - 1) carry_lds = before + inc;
        __syncthreads();
    }
}
__global__ void __launch_bounds__(kBlock) x_scan_write_kernel(const int64_t* __restrict__ first, int64_t npieces,
                                                              const int64_t* __restrict__ sums, int64_t* __restrict__ padded) {
    __shared__ long long wsum[kBlock / kWave];
    const int64_t g0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * kXScanPer;
    long long len[kXScanPer], mine = 0;
    for (int k = 0; k < kXScanPer; ++k) {
        len[k] = g0 + k < npieces ? x_padded_len(first, g0 + k) : 0;
        mine += len[k];
    }
    long long inc = mine;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    for (int off = 1; off < kWave; off <<= 1) {
        const long long t = __shfl_up(inc, off, kWave);
        if (lane >= off) inc += t;
    }
    if (lane == kWave - 1) wsum[wave] = inc;
    __syncthreads();
    long long at = sums[blockIdx.x] + inc - mine;
    for (int w = 0; w < wave; ++w) at += wsum[w];
    for (int k = 0; k < kXScanPer; ++k) {
        if (g0 + k < npieces) padded[g0 + k] = at;
        at += len[k];
        if (g0 + k == npieces - 1) padded[npieces] = at;
    }
}

// The entries: sorted edge e of piece g goes to padded[g] + (e - first[g]).
__global__ void __launch_bounds__(kBlock) x_entries_kernel(const uint64_t* __restrict__ keys, int64_t M, int bbits,
                                                           int64_t nrb, const int64_t* __restrict__ first,
                                                           const int64_t* __restrict__ padded,
                                                           uint16_t* __restrict__ x_src, uint16_t* __restrict__ x_row) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < M; e += stride) {
        const uint64_t k = keys[e];
        const int64_t g = x_piece_of(k, bbits, nrb);
        const int64_t pos = padded[g] + (e - first[g]);
        x_src[pos] = (uint16_t)((k >> kTileRowBits) & ((1u << kXSrcBits) - 1u));
        x_row[pos] = (uint16_t)(k & kTileRowMask);
    }
}
// The padding at the end of every piece.
__global__ void __launch_bounds__(kBlock) x_padding_kernel(int64_t npieces, const int64_t* __restrict__ first,
                                                           const int64_t* __restrict__ padded,
                                                           uint16_t* __restrict__ x_src, uint16_t* __restrict__ x_row) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t g = (int64_t)blockIdx.x * kBlock + threadIdx.x; g < npieces; g += stride)
        for (int64_t pos = padded[g] + (first[g + 1] - first[g]); pos < padded[g + 1]; ++pos) {
            x_src[pos] = (uint16_t)kXPad;
            x_row[pos] = 0;
        }
}
// Per row block b (one thread each; at step c the threads of a wavefront read neighbouring pieces):
// where its piece of every chunk starts, how many vectors of the block lie in earlier chunks, and
// the edges that end in the block.
__global__ void __launch_bounds__(kBlock) x_tables_kernel(int64_t nrb, int nch, const int64_t* __restrict__ first,
                                                          const int64_t* __restrict__ padded,
                                                          uint32_t* __restrict__ x_start, uint32_t* __restrict__ x_prefix,
                                                          int64_t* __restrict__ block_edges) {
    const int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (b >= nrb) return;
    uint32_t vecs = 0;
    int64_t edges = 0;
    for (int c = 0; c < nch; ++c) {
        const int64_t g = (int64_t)c * nrb + b;
        x_start[b * nch + c] = (uint32_t)(padded[g] >> 2);
        x_prefix[b * (nch + 1) + c] = vecs;
        vecs += (uint32_t)((padded[g + 1] - padded[g]) >> 2);
        edges += first[g + 1] - first[g];
    }
    x_prefix[b * (nch + 1) + nch] = vecs;
    block_edges[b] = edges;
}
__global__ void x_chunk_first_kernel(int64_t nrb, int nch, const int64_t* __restrict__ padded, int64_t* __restrict__ chunk_first) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c <= nch) chunk_first[c] = padded[(int64_t)c * nrb];
}
// block_first[b] = sum of counts[0 .. b), b <= nrb, by one workgroup (counts sits in block_first[1 ..]).
__global__ void __launch_bounds__(kBlock) block_first_kernel(int64_t* __restrict__ block_first, int64_t nrb) {
    __shared__ long long wsum[kBlock / kWave];
    __shared__ long long carry_lds;
    if (threadIdx.x == 0) { carry_lds = 0; }
    __syncthreads();
    for (int64_t base = 0; base < nrb; base += kBlock) {
        const int64_t i = base + threadIdx.x;
        const long long v = i < nrb ? block_first[i + 1] : 0;
        long long inc = v;
        const int lane = lane_id(), wave = threadIdx.x >> 6;
        for (int off = 1; off < kWave; off <<= 1) {
            const long long t = __shfl_up(inc, off, kWave);
            if (lane >= off) inc += t;
        }
        if (lane == kWave - 1) wsum[wave] = inc;
        __syncthreads();
        long long before = carry_lds;
        for (int w = 0; w < wave; ++w) before += wsum[w];
        __syncthreads();
        if (i < nrb) block_first[i + 1] = before + inc;          // inclusive: the prefix of b + 1
        if (threadIdx.x == kBlock - 1) carry_lds = before + inc;
        __syncthreads();
    }
    if (threadIdx.x == 0) block_first[0] = 0;
}

// Reads the arrays back the way the propagation kernels do: every entry that is not padding must
// be an edge of the CSR (found in the row of its source), lie in the piece that holds it, and the
// entries that are not padding must number M; the per-row-block tables must agree with the pieces'
// offsets.  A kernel that walks the structure afterwards never sees a source or a row out of range.
__global__ void __launch_bounds__(kBlock) x_verify_kernel(int64_t N, int64_t nrb, int nch, const int64_t* __restrict__ rowptr,
                                                          const int32_t* __restrict__ col,
                                                          const int64_t* __restrict__ padded, int64_t entries,
                                                          const uint16_t* __restrict__ x_src, const uint16_t* __restrict__ x_row,
                                                          const uint32_t* __restrict__ x_start, const uint32_t* __restrict__ x_prefix,
                                                          unsigned long long* __restrict__ real, int* __restrict__ bad) {
    __shared__ int lds[4];
    const int64_t npieces = nrb * nch;
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    int mine = 0;
    for (int64_t pos = (int64_t)blockIdx.x * kBlock + threadIdx.x; pos < entries; pos += stride) {
        const uint32_t s = x_src[pos];
        if (s & kXPad) continue;
        int64_t lo = 0, hi = npieces - 1;                       // last piece g with padded[g] <= pos
        while (lo < hi) {
            const int64_t mid = (lo + hi + 1) >> 1;
            if (padded[mid] <= pos) lo = mid; else hi = mid - 1;
        }
        const int64_t c = lo / nrb, b = lo - c * nrb;
        const int64_t v = (c << kXSrcBits) | s, u = (b << kTileRowBits) | x_row[pos];
        bool ok = pos < padded[lo + 1] && v < N && u < N && x_row[pos] <= kTileRowMask;
        if (ok) {
            int64_t a = rowptr[v], e = rowptr[v + 1];
            ok = false;
            while (a < e) {
                const int64_t mid = (a + e) >> 1;
                const int64_t w = col[mid];
                if (w == u) { ok = true; break; }
                if (w < u) a = mid + 1; else e = mid;
            }
        }
        if (!ok) *bad = 1;
        ++mine;
    }
    const int total = block_reduce_sum(mine, lds);
    if (threadIdx.x == 0 && total) atomicAdd(real, (unsigned long long)total);
    for (int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x; t < npieces; t += stride) {
        const int64_t b = t / nch, c = t - b * nch, g = c * nrb + b;
        const bool ok = (int64_t)x_start[t] * 4 == padded[g] &&
                        (int64_t)(x_prefix[b * (nch + 1) + c + 1] - x_prefix[b * (nch + 1) + c]) * 4 == padded[g + 1] - padded[g] &&
                        (c > 0 || x_prefix[b * (nch + 1)] == 0) && (padded[g] & 3) == 0;
        if (!ok) *bad = 1;
    }
}

struct XBuild {               // temporaries of build_chunked, freed on every path
    uint64_t *ka = nullptr, *kb = nullptr;
    int64_t *first = nullptr, *padded = nullptr, *sums = nullptr;
    unsigned long long* real = nullptr;
    int* bad = nullptr;
    ~XBuild() {
        (void)hipFree(ka); (void)hipFree(kb); (void)hipFree(first); (void)hipFree(padded); (void)hipFree(sums);
        (void)hipFree(real); (void)hipFree(bad);
    }
};

// The edges sorted by (chunk of sources, row block) with padded pieces, and the tables of both walks.
static int build_chunked(spp_ctx* ctx, spp_graph* g) {
    hipStream_t st = ctx->stream;
    const int64_t N = g->N, M = g->M;
    const int grid = ctx->num_cu * 8;
    const int nch = (int)((N + ((int64_t)1 << kXSrcBits) - 1) >> kXSrcBits);
    const int64_t nrb = (N + ((int64_t)1 << kTileRowBits) - 1) >> kTileRowBits;
    int bbits = 1, cbits = 1;
    while (((int64_t)1 << bbits) < nrb) ++bbits;
    while (((int64_t)1 << cbits) < nch) ++cbits;
    const int64_t npieces = nrb * nch;
    SPP_CHECK(M + 3 * npieces < ((int64_t)1 << 34), SPP_E_ARG, "chunked layout: %lld edges in %lld pieces exceed 2^32 vectors",
              (long long)M, (long long)npieces);
    g->tile_rbits = kTileRowBits; g->nrb = nrb; g->x_nch = nch;
    SPP_HIP(hipMalloc(&g->block_first, (size_t)(nrb + 1) * sizeof(int64_t)));
    SPP_HIP(hipMalloc(&g->x_chunk_first, (size_t)(nch + 1) * sizeof(int64_t)));
    SPP_HIP(hipMalloc(&g->x_start, (size_t)npieces * sizeof(uint32_t)));
    SPP_HIP(hipMalloc(&g->x_prefix, (size_t)nrb * (nch + 1) * sizeof(uint32_t)));
    XBuild t;
    SPP_HIP(hipMalloc(&t.first, (size_t)(npieces + 1) * sizeof(int64_t)));
    SPP_HIP(hipMalloc(&t.padded, (size_t)(npieces + 1) * sizeof(int64_t)));
    const int64_t nsum = (npieces + (int64_t)kBlock * kXScanPer - 1) / ((int64_t)kBlock * kXScanPer);
    SPP_HIP(hipMalloc(&t.sums, (size_t)(nsum + 1) * sizeof(int64_t)));
    SPP_HIP(hipMalloc(&t.real, sizeof(unsigned long long)));
    SPP_HIP(hipMalloc(&t.bad, sizeof(int)));
    SPP_HIP(hipMalloc(&t.ka, (size_t)(M > 0 ? M : 1) * sizeof(uint64_t)));
    SPP_HIP(hipMalloc(&t.kb, (size_t)(M > 0 ? M : 1) * sizeof(uint64_t)));
    uint64_t* sorted = t.ka;
    fill_i64_kernel<<<grid, kBlock, 0, st>>>(t.first, npieces + 1, M);
    if (M > 0) {
        x_keys_kernel<<<grid, kBlock, 0, st>>>(N, g->rowptr, g->col, bbits, t.ka);
        constexpr int lo_bits = kXSrcBits + kTileRowBits;
        SPP_TRY(radix_sort_u64(ctx, t.ka, t.kb, M, lo_bits, lo_bits + bbits + cbits, &sorted));
        x_bounds_kernel<<<grid, kBlock, 0, st>>>(sorted, M, bbits, nrb, t.first);
    }
    x_scan_sums_kernel<<<(unsigned)nsum, kBlock, 0, st>>>(t.first, npieces, t.sums);
    x_scan_top_kernel<<<1, kBlock, 0, st>>>(t.sums, nsum);
    x_scan_write_kernel<<<(unsigned)nsum, kBlock, 0, st>>>(t.first, npieces, t.sums, t.padded);
    int64_t entries = 0;
    SPP_HIP(hipMemcpyAsync(&entries, t.padded + npieces, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    SPP_HIP(hipStreamSynchronize(st));
    SPP_CHECK(entries >= M && entries <= M + 3 * npieces && (entries & 3) == 0, SPP_E_HIP,
              "chunked layout: %lld entries for %lld edges in %lld pieces", (long long)entries, (long long)M, (long long)npieces);
    g->x_entries = entries;
    SPP_HIP(hipMalloc(&g->x_src, (size_t)(entries > 0 ? entries : 4) * sizeof(uint16_t)));
    SPP_HIP(hipMalloc(&g->x_row, (size_t)(entries > 0 ? entries : 4) * sizeof(uint16_t)));
    if (M > 0) x_entries_kernel<<<grid, kBlock, 0, st>>>(sorted, M, bbits, nrb, t.first, t.padded, g->x_src, g->x_row);
    x_padding_kernel<<<grid, kBlock, 0, st>>>(npieces, t.first, t.padded, g->x_src, g->x_row);
    x_tables_kernel<<<(unsigned)((nrb + kBlock - 1) / kBlock), kBlock, 0, st>>>(nrb, nch, t.first, t.padded, g->x_start,
                                                                                g->x_prefix, g->block_first + 1);
    block_first_kernel<<<1, kBlock, 0, st>>>(g->block_first, nrb);
    x_chunk_first_kernel<<<(unsigned)((nch + 1 + kBlock - 1) / kBlock), kBlock, 0, st>>>(nrb, nch, t.padded, g->x_chunk_first);
    SPP_HIP(hipMemsetAsync(t.real, 0, sizeof(unsigned long long), st));
    SPP_HIP(hipMemsetAsync(t.bad, 0, sizeof(int), st));
    x_verify_kernel<<<grid, kBlock, 0, st>>>(N, nrb, nch, g->rowptr, g->col, t.padded, entries, g->x_src, g->x_row,
                                             g->x_start, g->x_prefix, t.real, t.bad);
    unsigned long long real = 0;
    int bad = 0;
    SPP_HIP(hipMemcpyAsync(&real, t.real, sizeof(real), hipMemcpyDeviceToHost, st));
    SPP_HIP(hipMemcpyAsync(&bad, t.bad, sizeof(bad), hipMemcpyDeviceToHost, st));
    SPP_HIP(hipStreamSynchronize(st));
    SPP_HIP(hipGetLastError());
    SPP_CHECK(bad == 0 && (int64_t)real == M, SPP_E_HIP,
              "chunked layout: the structure does not read back as the edges it was built from (%llu of %lld entries)",
              real, (long long)M);
    return SPP_OK;
}

}  // namespace spp

extern "C" int spp_graph_create(spp_ctx* ctx, int64_t N, int64_t M, const int64_t* d_rowptr,
                                const int32_t* d_col, uint32_t flags, spp_graph** out) {
    SPP_CHECK(ctx && out, SPP_E_ARG, "spp_graph_create: null argument");
    *out = nullptr;
    SPP_CHECK(N > 0 && N <= 0x7FFFFFFFll, SPP_E_ARG, "spp_graph_create: N = %lld out of range (int32 ids)", (long long)N);
    SPP_CHECK(M >= 0 && M < 0xFFFFFFFFll, SPP_E_ARG, "spp_graph_create: M = %lld out of range", (long long)M);
    SPP_CHECK(d_rowptr && (d_col || M == 0), SPP_E_ARG, "spp_graph_create: null CSR array");
    SPP_HIP(hipSetDevice(ctx->device));
    // the CSR must really describe M edges
    int64_t ends[2] = {-1, -1};
    SPP_HIP(hipMemcpy(&ends[0], d_rowptr, sizeof(int64_t), hipMemcpyDeviceToHost));
    SPP_HIP(hipMemcpy(&ends[1], d_rowptr + N, sizeof(int64_t), hipMemcpyDeviceToHost));
    SPP_CHECK(ends[0] == 0 && ends[1] == M, SPP_E_ARG, "spp_graph_create: rowptr[0] = %lld, rowptr[N] = %lld, M = %lld",
              (long long)ends[0], (long long)ends[1], (long long)M);
    spp_graph* g = new (std::nothrow) spp_graph();
    SPP_CHECK(g != nullptr, SPP_E_OOM, "spp_graph_create: out of host memory");
    g->device = ctx->device; g->N = N; g->M = M; g->rowptr = d_rowptr; g->col = d_col;
    {
        int* d_bad = nullptr;
        int bad = 0;
        hipError_t e = hipMalloc(&d_bad, sizeof(int));
        if (e == hipSuccess) e = hipMemsetAsync(d_bad, 0, sizeof(int), ctx->stream);
        if (e == hipSuccess) {
            spp::validate_csr_kernel<<<ctx->num_cu * 8, spp::kBlock, 0, ctx->stream>>>(N, M, d_rowptr, d_col, d_bad);
            e = hipMemcpyAsync(&bad, d_bad, sizeof(int), hipMemcpyDeviceToHost, ctx->stream);
        }
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (d_bad) (void)hipFree(d_bad);
        if (e != hipSuccess || bad) {
            if (e != hipSuccess) spp::set_error("spp_graph_create: %s", hipGetErrorString(e));
            else spp::set_error("spp_graph_create: rowptr is not monotone within [0, M] or a column id lies outside [0, N)");
            delete g;
            return e != hipSuccess ? SPP_E_HIP : SPP_E_ARG;
        }
    }
    if (flags & SPP_GRAPH_IN_LISTS) {
        // which layout: gathering y per edge pays while y stays in the caches (see spp_vip.hip)
        const bool chunked = (flags & SPP_GRAPH_CHUNKED) != 0 || N > spp::kChunkedAboveVertices;
        int rc = chunked ? spp::build_chunked(ctx, g) : spp::build_tiles(ctx, g);
        if (rc != SPP_OK) { spp_graph_destroy(g); return rc; }
        g->has_in = true;
        g->has_x = chunked;
    }
    *out = g;
    return SPP_OK;
}

extern "C" void spp_graph_destroy(spp_graph* g) {
    if (!g) return;
    if (hipSetDevice(g->device) != hipSuccess) { (void)hipGetLastError(); delete g; return; }   // runtime already shut down
    (void)hipDeviceSynchronize();      // work that still reads the row blocks may be in flight
    if (g->t_edge) (void)hipFree(g->t_edge);
    if (g->tile_first) (void)hipFree(g->tile_first);
    if (g->block_first) (void)hipFree(g->block_first);
    if (g->x_src) (void)hipFree(g->x_src);
    if (g->x_row) (void)hipFree(g->x_row);
    if (g->x_chunk_first) (void)hipFree(g->x_chunk_first);
    if (g->x_start) (void)hipFree(g->x_start);
    if (g->x_prefix) (void)hipFree(g->x_prefix);
    delete g;
}
