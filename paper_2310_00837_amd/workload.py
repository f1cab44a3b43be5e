"""Seeded synthetic workloads shaped after the paper's datasets (Table 1, Sec. 4.1).

This module only *produces inputs*: power-law CSR graphs, procedural feature
rows, a hotness order, train splits, seed batches and per-batch RNG seeds.  It
holds none of the sampling / dedup / cache / gather arithmetic; both the CPU
oracle's tests and the GPU library consume the arrays it returns.  All
randomness comes from one integer seed through a 64-bit counter hash, written
with torch integer ops so the same code runs on the CPU (small workloads) and
on the GPU (the 10^8-node workloads, generated where they are used).

The five workloads stand in for public datasets that are not available here:
workloads 2 and 4 copy the vertex/edge/feature shape of the paper's PA row
(111 M vertices, 1.6 B edges, fp32 dim 128), workload 3 the dim-1024
"manually generated features" setting of its UK/CL/LD rows.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Callable, List, Optional, Tuple

import torch

_M64 = (1 << 64) - 1


def _s64(c: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 holds for it."""
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


_C1 = _s64(0x9E3779B97F4A7C15)
_C2 = _s64(0xBF58476D1CE4E5B9)
_C3 = _s64(0x94D049BB133111EB)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """64-bit finaliser (xor-shift-multiply, the SplitMix64 output function)."""
    z = x + _C1
    z = (z ^ _lsr(z, 30)) * _C2
    z = (z ^ _lsr(z, 27)) * _C3
    return z ^ _lsr(z, 31)


def mix64_int(x: int) -> int:
    z = (x + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, tag: str) -> int:
    """Sub-stream key for a purpose tag, as a signed int64 value."""
    k = seed & _M64
    for ch in tag.encode():
        k = mix64_int(k ^ ch)
    return _s64(k)


def hash_u64(seed: int, tag: str, idx: torch.Tensor) -> torch.Tensor:
    """hash(seed, tag, idx) as int64 bit patterns; idx is an int64 tensor."""
    return mix64(mix64(idx + stream_key(seed, tag)))


def uniform01(seed: int, tag: str, idx: torch.Tensor) -> torch.Tensor:
    """Uniform doubles in [0, 1) with 53 random bits."""
    return _lsr(hash_u64(seed, tag, idx), 11).to(torch.float64) * (2.0 ** -53)


def hash_permutation(seed: int, tag: str, n: int, device) -> torch.Tensor:
    """A permutation of 0..n-1: argsort of per-index hashes (stable)."""
    h = hash_u64(seed, tag, torch.arange(n, dtype=torch.int64, device=device))
    return torch.sort(h, stable=True).indices


# --------------------------------------------------------------------------
# features


def feature_rows(seed: int, ids: torch.Tensor, dim: int, dtype: torch.dtype) -> torch.Tensor:
    """Procedural feature rows feat(id, col), uniform on [-1, 1), exactly
    representable in `dtype` (fp32: 24 random bits, fp16: 11 random bits)."""
    assert dim <= 4096
    ids = ids.to(torch.int64)
    cols = torch.arange(dim, dtype=torch.int64, device=ids.device)
    ctr = (ids[:, None] << 12) | cols[None, :]
    h = _lsr(hash_u64(seed, "feat", ctr), 32)          # 32 random bits
    if dtype == torch.float32:
        return (_lsr(h, 8).to(torch.float32) * (2.0 ** -23)) - 1.0
    if dtype == torch.float16:
        return ((_lsr(h, 21).to(torch.float32) * (2.0 ** -10)) - 1.0).to(torch.float16)
    raise ValueError("dtype must be float32 or float16")


def fill_rows(dst: torch.Tensor, seed: int, ids: torch.Tensor, chunk_elems: int = 1 << 26,
              progress: Optional[Callable[[str], None]] = None) -> None:
    """dst[i, :] = feat(ids[i], :) in chunks; dst may live on another device
    than ids (e.g. pinned host memory filled from GPU-generated chunks)."""
    n, dim = dst.shape
    rows = max(1, chunk_elems // dim)
    for r0 in range(0, n, rows):
        r1 = min(n, r0 + rows)
        blk = feature_rows(seed, ids[r0:r1], dim, dst.dtype)
        dst[r0:r1].copy_(blk)
        if progress is not None and (r0 // rows) % 64 == 0:
            progress(f"fill_rows {r1}/{n}")


# --------------------------------------------------------------------------
# graph


def _power_law_params(n: int, e: float, gamma: float) -> Tuple[float, float, float]:
    """Weights w_i = c (i + i0)^(-alpha), alpha = 1/(gamma-1), with
    w_0 = sqrt(E) and sum_i w_i = E (integral approximation).  Returns
    (alpha, i0, c)."""
    alpha = 1.0 / (gamma - 1.0)
    wmax = math.sqrt(e)
    q = 1.0 - alpha

    def total(i0: float) -> float:
        c = wmax * i0 ** alpha
        return c * ((n + i0) ** q - i0 ** q) / q

    lo, hi = 1e-9, float(n) * 1e3
    for _ in range(200):                   # total(i0) grows with i0
        mid = math.sqrt(lo * hi)
        if total(mid) < e:
            lo = mid
        else:
            hi = mid
    i0 = math.sqrt(lo * hi)
    return alpha, i0, wmax * i0 ** alpha


def chung_lu_csr(seed: int, n: int, e_target: int, gamma: float, device,
                 edge_chunk: int = 1 << 27,
                 progress: Optional[Callable[[str], None]] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Directed Chung-Lu graph with power-law expected degrees (exponent
    gamma).  Row v lists the nodes that can be sampled as neighbours of v.
    Rows are sorted, duplicate-free and without self loops, so the edge count
    is close to (a little below) e_target.  Returns (offsets int64[n+1],
    indices int32[E])."""
    alpha, i0, c = _power_law_params(n, float(e_target), gamma)
    q = 1.0 - alpha
    dev = torch.device(device)
    ar = torch.arange(n, dtype=torch.int64, device=dev)
    # out-degree: weight index of node v is perm_out[v]; stochastic rounding of w
    perm_out = hash_permutation(seed, "perm_out", n, dev)
    w = c * (perm_out.to(torch.float64) + i0) ** (-alpha)
    deg = torch.floor(w).to(torch.int64) + (uniform01(seed, "deg_round", ar) < (w - torch.floor(w))).to(torch.int64)
    del w, perm_out
    perm_in = hash_permutation(seed, "perm_in", n, dev).to(torch.int32)
    raw_off = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    raw_off[1:] = torch.cumsum(deg, 0)
    e_raw = int(raw_off[-1].item())
    a_hi = (n + i0) ** q
    a_lo = i0 ** q
    inv_q = 1.0 / q
    new_deg = torch.zeros(n, dtype=torch.int64, device=dev)
    out_chunks: List[torch.Tensor] = []
    # process whole rows in chunks of about edge_chunk raw edges
    r0 = 0
    raw_off_cpu_probe = raw_off  # searched on device
    while r0 < n:
        target = int(raw_off[r0].item()) + edge_chunk
        r1 = int(torch.searchsorted(raw_off_cpu_probe, torch.tensor([target], device=dev), right=True).item()) - 1
        r1 = max(r0 + 1, min(n, r1))
        e0, e1 = int(raw_off[r0].item()), int(raw_off[r1].item())
        if e1 > e0:
            eidx = torch.arange(e0, e1, dtype=torch.int64, device=dev)
            rows = torch.searchsorted(raw_off[r0:r1 + 1], eidx, right=True) - 1 + r0
            u = uniform01(seed, "nbr", eidx)
            x = (a_lo + u * (a_hi - a_lo)) ** inv_q - i0
            widx = torch.clamp(x.to(torch.int64), 0, n - 1)
            del u, x, eidx
            nbr = perm_in[widx].to(torch.int64)
            del widx
            keep = nbr != rows
            key = (rows * n + nbr)[keep]
            del rows, nbr, keep
            key = torch.unique(key)                # sorted: by row, then by neighbour
            krow = key // n
            out_chunks.append((key - krow * n).to(torch.int32))
            new_deg += torch.bincount(krow, minlength=n)
            del key, krow
        if progress is not None:
            progress(f"chung_lu rows {r1}/{n}")
        r0 = r1
    offsets = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    offsets[1:] = torch.cumsum(new_deg, 0)
    indices = torch.cat(out_chunks) if out_chunks else torch.zeros(0, dtype=torch.int32, device=dev)
    assert indices.numel() == int(offsets[-1].item()) and e_raw >= indices.numel()
    return offsets, indices


def in_degree_order(indices: torch.Tensor, n: int) -> torch.Tensor:
    """Nodes by in-degree (occurrences in `indices`) descending, ties by
    ascending node ID.  int32[n]."""
    indeg = torch.zeros(n, dtype=torch.int64, device=indices.device)
    step = 1 << 28
    for s in range(0, indices.numel(), step):
        indeg += torch.bincount(indices[s:s + step].to(torch.int64), minlength=n)
    return torch.sort(indeg, descending=True, stable=True).indices.to(torch.int32)


# --------------------------------------------------------------------------
# workload table (benchmark configs, 0-based)


@dataclass
class WorkloadSpec:
    name: str
    n_nodes: int
    n_edges: int
    dim: int
    dtype: torch.dtype
    batch: int
    fanouts: List[int]
    train_frac: float
    hbm: Tuple[str, float]          # ("frac", fraction of N) or ("bytes", bytes)
    host: Tuple[str, float]         # ("frac", ...), ("bytes", ...) or ("half_rest", 0)
    seeds: str = "split"            # "split" or "zipf"
    gamma: float = 2.1

    @property
    def row_bytes(self) -> int:
        return self.dim * (4 if self.dtype == torch.float32 else 2)

    def tier_rows(self, n_nodes: Optional[int] = None) -> Tuple[int, int, int]:
        n = self.n_nodes if n_nodes is None else n_nodes

        def rows(kind: str, val: float, rest: int) -> int:
            if kind == "frac":
                r = int(math.floor(val * n + 1e-9))
            elif kind == "bytes":
                r = int(val) // self.row_bytes
            elif kind == "half_rest":
                r = rest // 2
            else:
                raise ValueError(kind)
            return max(0, min(r, rest))

        n_hbm = rows(self.hbm[0], self.hbm[1], n)
        n_host = rows(self.host[0], self.host[1], n - n_hbm)
        return n_hbm, n_host, n - n_hbm - n_host


def spec(cfg: int, hbm_frac: Optional[float] = None) -> WorkloadSpec:
    f32, f16 = torch.float32, torch.float16
    if cfg == 0:
        return WorkloadSpec("cfg0-tiny", 10_000, 100_000, 64, f32, 128, [5, 5], 0.10, ("frac", 0.10), ("frac", 0.20))
    if cfg == 1:
        return WorkloadSpec("cfg1-medium", 1_000_000, 15_000_000, 128, f32, 1024, [10, 10], 0.10, ("frac", 0.10), ("frac", 0.30))
    if cfg == 2:
        return WorkloadSpec("cfg2-large", 111_000_000, 1_600_000_000, 128, f32, 1024, [25, 10], 0.01, ("bytes", 20e9), ("bytes", 30e9))
    if cfg == 3:
        return WorkloadSpec("cfg3-wide", 50_000_000, 1_000_000_000, 1024, f16, 1024, [10, 10, 10], 0.01, ("bytes", 64e9), ("bytes", 24e9))
    if cfg == 4:
        p = 0.25 if hbm_frac is None else hbm_frac
        return WorkloadSpec(f"cfg4-sweep-hbm{int(round(p * 100))}", 111_000_000, 1_600_000_000, 128, f32, 1024, [25, 10], 0.01,
                            ("frac", p), ("half_rest", 0.0), seeds="zipf")
    raise ValueError("cfg must be 0..4")


@dataclass
class Graph:
    seed: int
    n_nodes: int
    offsets: torch.Tensor       # int64[n+1]
    indices: torch.Tensor       # int32[E]
    order: torch.Tensor         # int32[n], hotness order (in-degree descending)
    perm_seed: torch.Tensor = field(repr=False, default=None)   # int64[n], permutation used for splits

    @property
    def n_edges(self) -> int:
        return int(self.indices.numel())


def make_graph(sp: WorkloadSpec, seed: int, device, scale: float = 1.0,
               progress: Optional[Callable[[str], None]] = None) -> Graph:
    """`scale` < 1 shrinks nodes and edges together (used by CPU-side tests of
    the generator itself); the workloads proper use scale = 1."""
    n = max(16, int(sp.n_nodes * scale))
    e = max(16, int(sp.n_edges * scale))
    offsets, indices = chung_lu_csr(seed, n, e, sp.gamma, device, progress=progress)
    order = in_degree_order(indices, n)
    perm = hash_permutation(seed, "perm_split", n, torch.device(device))
    return Graph(seed, n, offsets, indices, order, perm)


def batch_rng_seed(seed: int, batch_index: int) -> int:
    """The 64-bit rng_seed the sampler receives for batch `batch_index`."""
    return mix64_int(mix64_int((seed & _M64) ^ 0x62617463685F7267) + batch_index)


def seed_batch(sp: WorkloadSpec, g: Graph, batch_index: int, epoch: int = 0) -> torch.Tensor:
    """int32[batch] seed nodes of one mini-batch.
    "split": train = first floor(train_frac * N) entries of a seeded permutation;
    an epoch is a seeded shuffle of train cut into consecutive batches (seeds
    distinct within a batch; the list wraps around at the end of the epoch).
    "zipf": seed = perm[k-1], k = min(N, floor((N+1)^u)), u uniform on [0,1):
    the continuous inverse CDF of a Zipf law with s = 1; duplicates are kept."""
    n = g.n_nodes
    dev = g.perm_seed.device
    b = min(sp.batch, n)
    if sp.seeds == "split":
        n_train = max(b, int(math.floor(sp.train_frac * n)))
        n_train = min(n_train, n)
        train = g.perm_seed[:n_train]
        shuf = hash_permutation(g.seed + 7919 * (epoch + 1), "epoch_shuffle", n_train, dev)
        pos = (torch.arange(b, dtype=torch.int64, device=dev) + batch_index * b) % n_train
        return train[shuf[pos]].to(torch.int32)
    if sp.seeds == "zipf":
        idx = torch.arange(b, dtype=torch.int64, device=dev) + (batch_index * b) + (epoch << 40)
        u = uniform01(g.seed, "zipf", idx)
        k = torch.clamp(torch.floor(torch.exp(u * math.log(n + 1.0))).to(torch.int64), 1, n)
        return g.perm_seed[k - 1].to(torch.int32)
    raise ValueError(sp.seeds)


@dataclass
class Tiers:
    """Feature tables in rank order (row r of the concatenation = feat(order[r]))."""
    n_hbm: int
    n_host: int
    n_rest: int
    row_bytes: int
    hbm: torch.Tensor          # [max(n_hbm,1), dim] on the GPU
    host: torch.Tensor         # [max(n_host,1), dim] pinned host memory
    standin: torch.Tensor      # [max(n_rest,1), dim] pinned host memory (storage stand-in)


def make_tiers(sp: WorkloadSpec, g: Graph, device, progress: Optional[Callable[[str], None]] = None,
               pinned_empty: Optional[Callable] = None) -> Tiers:
    """Fill the three tier tables directly in rank order; the full feature table is never
    materialised.  `device` is where the HBM tier lives and where rows are generated.
    pinned_empty(shape, dtype) -> tensor allocates the two host tables (default: torch's
    pinned allocator, which rounds sizes up to a power of two)."""
    n_hbm, n_host, n_rest = sp.tier_rows(g.n_nodes)
    dev = torch.device(device)
    order = g.order.to(dev)
    pin = dev.type == "cuda"
    hbm = torch.empty((max(n_hbm, 1), sp.dim), dtype=sp.dtype, device=dev)
    if pinned_empty is None:
        def pinned_empty(shape, dtype):
            return torch.empty(shape, dtype=dtype, pin_memory=pin)
    host = pinned_empty((max(n_host, 1), sp.dim), sp.dtype)
    standin = pinned_empty((max(n_rest, 1), sp.dim), sp.dtype)
    fill_rows(hbm[:n_hbm], g.seed, order[:n_hbm], progress=progress)
    fill_rows(host[:n_host], g.seed, order[n_hbm:n_hbm + n_host], progress=progress)
    fill_rows(standin[:n_rest], g.seed, order[n_hbm + n_host:], progress=progress)
    return Tiers(n_hbm, n_host, n_rest, sp.row_bytes, hbm, host, standin)
