"""Seeded synthetic inputs shaped like the paper's workloads (Table 2, Table 3).

This module only makes inputs: graphs, partitions, training sets, minibatches and
feature rows.  It holds none of the method's arithmetic (no inclusion
probabilities, no sampling of neighbourhoods, no cache ranking) and is the one
module that both the CPU oracle's tests and the HIP path's tests draw from.

Everything is written with device-agnostic torch tensor ops so the same recipe
runs on the CPU (small cases, no GPU needed) and on the GPU (the cases with
10^8 vertices, which would take hours on the host).  A given (config, device
type) pair always produces the same arrays; whatever is produced is handed,
as the same arrays, to both the oracle and the HIP path.

Recipes
-------
graph "zipf_out": out-degree d(v) ~ truncated Zipf on [1, cap]; if the config
    fixes the exponent s the degrees are rescaled multiplicatively to the stated
    mean (floor 1), otherwise s is solved by bisection so that the truncated
    distribution has that mean.  Each edge's target is uniform inside the source's
    partition with probability `intra`, else uniform over the vertices outside
    it.  Self loops are dropped and every row is sorted and made unique.
graph "zipf_in": as above for the out-degrees (lightly skewed), but every vertex
    carries a popularity weight ~ truncated Zipf(s_in) on [1, pop_cap] and targets
    are drawn in proportion to that weight inside the chosen id range, so the
    in-degree distribution is heavy-tailed as in a citation graph.
graph "rmat": recursive-matrix edges (a, b, c, d) at the given scale and edge
    factor, ids permuted by a seeded permutation, self loops dropped, rows
    sort-uniqued.
partitions: K contiguous id ranges, bounds[k] = floor(k*N/K).
training set: exactly round(train_frac*N) vertices, uniform without replacement.
features: feat(seed, g, j) is a pure function of vertex id and column: the sum of
    twelve 16-bit uniforms from a 64-bit mixing hash, centred and scaled to unit
    variance (Irwin-Hall, a bounded stand-in for N(0,1)).  It uses only integer
    operations and one exact scaling, so any row can be regenerated bit-exactly on
    any device without holding the matrix.
minibatches: a seeded permutation of the partition's training vertices per epoch,
    cut into chunks of B (the last may be short).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional, Sequence, Tuple

import torch


@dataclasses.dataclass(frozen=True)
class WorkloadConfig:
    name: str
    N: int
    mean_degree: float
    degree_cap: int
    intra: float
    D: int
    dtype: str                      # "fp32" | "fp16" | "bf16"
    train_frac: float
    fanouts: Tuple[int, ...]
    B: int
    K: int
    alpha: float
    owned_partition: int = 0
    graph: str = "zipf_out"         # "zipf_out" | "zipf_in" | "rmat"
    zipf_s: Optional[float] = None  # fixed out-degree exponent (then degrees are rescaled)
    zipf_s_in: float = 1.8          # popularity exponent for "zipf_in"
    pop_cap: int = 100_000          # largest popularity weight for "zipf_in"
    rmat_scale: int = 0
    rmat_edge_factor: int = 0
    rmat_abcd: Tuple[float, float, float, float] = (0.57, 0.19, 0.19, 0.05)
    seed_graph: int = 1
    seed_feat: int = 2
    seed_train: int = 3
    seed_sampler: int = 4

    @property
    def L(self) -> int:
        return len(self.fanouts)

    @property
    def elem_bytes(self) -> int:
        return {"fp32": 4, "fp16": 2, "bf16": 2}[self.dtype]

    @property
    def torch_dtype(self) -> torch.dtype:
        return {"fp32": torch.float32, "fp16": torch.float16, "bf16": torch.bfloat16}[self.dtype]

    def bounds(self) -> Tuple[int, int]:
        k = self.owned_partition
        return (k * self.N) // self.K, ((k + 1) * self.N) // self.K

    def cache_capacity(self, alpha: Optional[float] = None) -> int:
        a = self.alpha if alpha is None else alpha
        return int(math.floor(a * float(self.N) / self.K))


TINY = WorkloadConfig("tiny", N=10_000, mean_degree=10.0, degree_cap=1_000, intra=0.70, D=32,
                      dtype="fp32", train_frac=0.10, fanouts=(15, 10, 5), B=256, K=4, alpha=0.10,
                      zipf_s=2.0)
MID = WorkloadConfig("mid", N=2_400_000, mean_degree=51.0, degree_cap=20_000, intra=0.75, D=100,
                     dtype="fp32", train_frac=0.08, fanouts=(15, 10, 5), B=1024, K=8, alpha=0.16)
LARGE = WorkloadConfig("large", N=111_000_000, mean_degree=29.0, degree_cap=50_000, intra=0.80,
                       D=128, dtype="fp16", train_frac=0.011, fanouts=(15, 10, 5), B=1024, K=8,
                       alpha=0.32)
WIDE = WorkloadConfig("wide", N=121_000_000, mean_degree=21.5, degree_cap=5_000, intra=0.70, D=768,
                      dtype="fp16", train_frac=1_100_000 / 121_000_000, fanouts=(25, 15), B=1024,
                      K=8, alpha=0.16, graph="zipf_in", zipf_s_in=1.8)
SKEW = WorkloadConfig("skew", N=1 << 27, mean_degree=16.0, degree_cap=0, intra=0.0, D=256,
                      dtype="bf16", train_frac=0.01, fanouts=(20, 15, 10), B=4096, K=16, alpha=0.5,
                      graph="rmat", rmat_scale=27, rmat_edge_factor=16)

CONFIGS = {c.name: c for c in (TINY, MID, LARGE, WIDE, SKEW)}


def scaled(cfg: WorkloadConfig, N: int, **kw) -> WorkloadConfig:
    """A copy of `cfg` with fewer vertices (same recipe), for parity cases the oracle finishes fast."""
    cap = min(cfg.degree_cap, max(8, N // (4 * cfg.K))) if cfg.degree_cap else 0
    rs = cfg.rmat_scale
    if cfg.graph == "rmat":
        rs = int(math.log2(N))
        N = 1 << rs
    pop = min(cfg.pop_cap, max(16, N // (64 * cfg.K)))
    args = dict(name=f"{cfg.name}@{N}", N=N, degree_cap=cap, rmat_scale=rs, pop_cap=pop)
    args.update(kw)
    return dataclasses.replace(cfg, **args)


# ----------------------------------------------------------------------------------------------
# helpers
# ----------------------------------------------------------------------------------------------

def _gen(device, *keys: int) -> torch.Generator:
    g = torch.Generator(device=device)
    s = 0x243F6A8885A308D3
    for k in keys:
        s = ((s ^ (int(k) & 0xFFFFFFFFFFFFFFFF)) * 0x9E3779B97F4A7C15 + 0x7F4A7C15) & 0x7FFFFFFFFFFFFFFF
    g.manual_seed(s)
    return g


def _truncated_zipf_mean(s: float, cap: int) -> float:
    k = torch.arange(1, cap + 1, dtype=torch.float64)
    w = k.pow(-s)
    return float((k * w).sum() / w.sum())


def _solve_zipf_exponent(mean: float, cap: int) -> float:
    lo, hi = 0.05, 6.0          # mean is decreasing in s
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        if _truncated_zipf_mean(mid, cap) > mean:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def _zipf_draw(u: torch.Tensor, s: float, cap: int) -> torch.Tensor:
    """Inverse-CDF draw of a truncated Zipf(s) on [1, cap] from uniforms u (float64 in [0,1))."""
    k = torch.arange(1, cap + 1, dtype=torch.float64, device=u.device)
    cdf = torch.cumsum(k.pow(-s), 0)
    cdf = cdf / cdf[-1]
    return (torch.searchsorted(cdf, u, right=False).clamp_(max=cap - 1) + 1).to(torch.int64)


def _out_degrees(cfg: WorkloadConfig, device) -> torch.Tensor:
    g = _gen(device, cfg.seed_graph, 11)
    u = torch.rand(cfg.N, generator=g, dtype=torch.float64, device=device)
    if cfg.zipf_s is not None:
        z = _zipf_draw(u, cfg.zipf_s, cfg.degree_cap)
        scale = cfg.mean_degree / _truncated_zipf_mean(cfg.zipf_s, cfg.degree_cap)
        d = torch.round(z.to(torch.float64) * scale).to(torch.int64)
    else:
        s = _solve_zipf_exponent(cfg.mean_degree, cfg.degree_cap)
        d = _zipf_draw(u, s, cfg.degree_cap)
    return d.clamp_(min=1, max=cfg.degree_cap)


def _part_bounds(cfg: WorkloadConfig, device) -> torch.Tensor:
    return torch.tensor([(k * cfg.N) // cfg.K for k in range(cfg.K + 1)], dtype=torch.int64, device=device)


def _rows_to_csr(src: torch.Tensor, tgt: torch.Tensor, row_lo: int, row_hi: int):
    """Drop self loops, sort-unique (src, tgt) pairs; return per-row counts and the column list."""
    keep = src != tgt
    key = (src[keep] << 32) | tgt[keep]
    key = torch.unique(key)            # sorted ascending, duplicates removed
    s = key >> 32
    col = (key & 0xFFFFFFFF).to(torch.int32)
    counts = torch.bincount(s - row_lo, minlength=row_hi - row_lo)
    return counts, col


def _edge_chunk_rows(deg: torch.Tensor, max_edges: int):
    """Cut [0,N) into consecutive row ranges of at most ~max_edges raw edges each."""
    csum = torch.cumsum(deg, 0)
    total = int(csum[-1])
    cuts = [0]
    nxt = max_edges
    while nxt < total:
        r = int(torch.searchsorted(csum, torch.tensor([nxt], device=deg.device))[0]) + 1
        r = max(r, cuts[-1] + 1)
        cuts.append(r)
        nxt = int(csum[r - 1]) + max_edges
    cuts.append(deg.numel())
    return [(a, b) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]


def _targets_partitioned(cfg, src, bounds, g, device, popcum: Optional[torch.Tensor]):
    n = src.numel()
    part = torch.bucketize(src, bounds[1:], right=True)
    lo = bounds[part]
    hi = bounds[part + 1]
    size = hi - lo
    u_sel = torch.rand(n, generator=g, device=device)
    u_pos = torch.rand(n, generator=g, dtype=torch.float64, device=device)
    intra = u_sel < cfg.intra
    if popcum is not None:
        # targets proportional to a per-vertex popularity weight; popcum[i] = sum of weights of
        # vertices < i (length N+1).  Intra: inside [lo,hi); inter: over the rest, skipping [lo,hi).
        w_lo, w_hi, w_all = popcum[lo], popcum[hi], popcum[-1]
        w_part = w_hi - w_lo
        x_in = w_lo + u_pos * w_part
        x_out = u_pos * (w_all - w_part)
        x_out = torch.where(x_out < w_lo, x_out, x_out + w_part)
        x = torch.where(intra, x_in, x_out)
        tgt = (torch.searchsorted(popcum, x, right=True) - 1).clamp_(min=0, max=cfg.N - 1)
        # rounding at a range edge may land one vertex outside the intended side; harmless
        return tgt
    rng = torch.where(intra, size, cfg.N - size)
    off = torch.minimum((u_pos * rng.to(torch.float64)).to(torch.int64), rng - 1)
    return torch.where(intra, lo + off, torch.where(off < lo, off, off + size))


def _popularity_cumsum(cfg: WorkloadConfig, device) -> torch.Tensor:
    """Per-vertex popularity weights ~ truncated Zipf(s_in) on [1, pop_cap], as a cumulative sum."""
    g = _gen(device, cfg.seed_graph, 15)
    u = torch.rand(cfg.N, generator=g, dtype=torch.float64, device=device)
    w = _zipf_draw(u, cfg.zipf_s_in, cfg.pop_cap).to(torch.float64)
    cum = torch.zeros(cfg.N + 1, dtype=torch.float64, device=device)
    torch.cumsum(w, 0, out=cum[1:])
    return cum


def _rmat_edges(cfg: WorkloadConfig, n_edges: int, g, device):
    a, b, c, _ = cfg.rmat_abcd
    src = torch.zeros(n_edges, dtype=torch.int64, device=device)
    dst = torch.zeros(n_edges, dtype=torch.int64, device=device)
    for _ in range(cfg.rmat_scale):
        u = torch.rand(n_edges, generator=g, device=device)
        sbit = (u >= a + b).to(torch.int64)                       # quadrants c, d: lower half
        dbit = (((u >= a) & (u < a + b)) | (u >= a + b + c)).to(torch.int64)  # quadrants b, d
        src = (src << 1) | sbit
        dst = (dst << 1) | dbit
    return src, dst


@dataclasses.dataclass
class Graph:
    N: int
    M: int
    rowptr: torch.Tensor   # int64[N+1]
    col: torch.Tensor      # int32[M]; rows ascending, unique, no self loops


def make_graph(cfg: WorkloadConfig, device="cpu", max_chunk_edges: int = 1 << 27) -> Graph:
    device = torch.device(device)
    N = cfg.N
    if cfg.graph == "rmat":
        return _make_rmat(cfg, device, max_chunk_edges)
    deg = _out_degrees(cfg, device)
    bounds = _part_bounds(cfg, device)
    popcum = _popularity_cumsum(cfg, device) if cfg.graph == "zipf_in" else None
    counts_all, cols = [], []
    for ci, (r0, r1) in enumerate(_edge_chunk_rows(deg, max_chunk_edges)):
        g = _gen(device, cfg.seed_graph, 12, ci)
        rows = torch.arange(r0, r1, dtype=torch.int64, device=device)
        src = torch.repeat_interleave(rows, deg[r0:r1])
        tgt = _targets_partitioned(cfg, src, bounds, g, device, popcum)
        counts, col = _rows_to_csr(src, tgt, r0, r1)
        counts_all.append(counts)
        cols.append(col)
        del src, tgt
    counts = torch.cat(counts_all)
    rowptr = torch.zeros(N + 1, dtype=torch.int64, device=device)
    torch.cumsum(counts, 0, out=rowptr[1:])
    col = torch.cat(cols) if len(cols) > 1 else cols[0]
    return Graph(N=N, M=int(col.numel()), rowptr=rowptr, col=col)


def _make_rmat(cfg: WorkloadConfig, device, max_chunk_edges: int) -> Graph:
    N = 1 << cfg.rmat_scale
    total = N * cfg.rmat_edge_factor
    perm = torch.randperm(N, generator=_gen(device, cfg.seed_graph, 13), device=device)
    keys = []
    done = 0
    ci = 0
    while done < total:
        n = min(max_chunk_edges, total - done)
        s, d = _rmat_edges(cfg, n, _gen(device, cfg.seed_graph, 14, ci), device)
        s, d = perm[s], perm[d]
        keep = s != d
        keys.append(torch.unique((s[keep] << 32) | d[keep]))
        done += n
        ci += 1
    key = torch.unique(torch.cat(keys)) if len(keys) > 1 else keys[0]
    src = key >> 32
    col = (key & 0xFFFFFFFF).to(torch.int32)
    counts = torch.bincount(src, minlength=N)
    rowptr = torch.zeros(N + 1, dtype=torch.int64, device=device)
    torch.cumsum(counts, 0, out=rowptr[1:])
    return Graph(N=N, M=int(col.numel()), rowptr=rowptr, col=col)


def make_training_set(cfg: WorkloadConfig, device="cpu") -> torch.Tensor:
    """All training vertices (sorted int32), exactly round(train_frac * N) of them."""
    device = torch.device(device)
    n = int(round(cfg.train_frac * cfg.N))
    perm = torch.randperm(cfg.N, generator=_gen(device, cfg.seed_train, 21), device=device)
    return torch.sort(perm[:n]).values.to(torch.int32)


def local_training_set(cfg: WorkloadConfig, train: torch.Tensor) -> torch.Tensor:
    lo, hi = cfg.bounds()
    return train[(train >= lo) & (train < hi)].contiguous()


def epoch_batches(cfg: WorkloadConfig, train_local: torch.Tensor, epoch: int):
    """Seeded permutation of the partition's training vertices, cut into chunks of B."""
    dev = train_local.device
    perm = torch.randperm(train_local.numel(), generator=_gen(dev, cfg.seed_sampler, 31, epoch), device=dev)
    shuffled = train_local[perm]
    return [shuffled[i:i + cfg.B].contiguous() for i in range(0, shuffled.numel(), cfg.B)]


# ----------------------------------------------------------------------------------------------
# features: pure function of (seed, vertex, column)
# ----------------------------------------------------------------------------------------------

def _i64(x: int) -> int:
    x &= 0xFFFFFFFFFFFFFFFF
    return x - (1 << 64) if x >= (1 << 63) else x


_MIX1 = _i64(0xBF58476D1CE4E5B9)
_MIX2 = _i64(0x94D049BB133111EB)
_GOLD = _i64(0x9E3779B97F4A7C15)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    x = (x ^ _lsr(x, 30)) * _MIX1
    x = (x ^ _lsr(x, 27)) * _MIX2
    return x ^ _lsr(x, 31)


def feature_rows(cfg: WorkloadConfig, ids: torch.Tensor) -> torch.Tensor:
    """Rows feat(seed_feat, g, 0..D-1) for the vertex ids given, in the config's storage type."""
    ids = ids.to(torch.int64)
    dev = ids.device
    j = torch.arange(cfg.D, dtype=torch.int64, device=dev)
    base = (ids[:, None] * cfg.D + j[None, :]) * 3 + _i64(cfg.seed_feat * 0x632BE59BD9B4E019)
    acc = torch.zeros(base.shape, dtype=torch.int64, device=dev)
    for w in range(3):
        h = _mix64((base + w) * _GOLD)
        for q in range(4):
            acc += _lsr(h, 16 * q) & 0xFFFF
    # twelve uniforms on {0..65535}: mean 12*32767.5, variance 12*(65536^2-1)/12 ~ 65536^2
    x = (acc - 393210).to(torch.float32) * (1.0 / 65536.0)
    return x.to(cfg.torch_dtype)


def feature_block(cfg: WorkloadConfig, lo: int, hi: int, device="cpu", chunk: int = 1 << 20,
                  out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Rows lo..hi-1, generated in chunks (into `out` if given, which may be pinned host memory)."""
    device = torch.device(device)
    if out is None:
        out = torch.empty((hi - lo, cfg.D), dtype=cfg.torch_dtype, device=device)
    for a in range(lo, hi, chunk):
        b = min(hi, a + chunk)
        rows = feature_rows(cfg, torch.arange(a, b, dtype=torch.int64, device=device))
        out[a - lo:b - lo].copy_(rows)
    return out


def remote_row_index(cfg: WorkloadConfig, g: torch.Tensor) -> torch.Tensor:
    """Row of vertex g in the remote store (the feature matrix with the owned range cut out)."""
    lo, hi = cfg.bounds()
    return torch.where(g < lo, g, g - (hi - lo))


def remote_ids(cfg: WorkloadConfig, a: int, b: int, device="cpu") -> torch.Tensor:
    """Vertex ids of remote-store rows a..b-1."""
    lo, hi = cfg.bounds()
    r = torch.arange(a, b, dtype=torch.int64, device=device)
    return torch.where(r < lo, r, r + (hi - lo))
