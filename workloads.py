"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU library's tests/bench.

This module produces *inputs only*: latency / bandwidth matrices, message sizes and candidate
permutations. It holds none of the cost model's arithmetic (no weights, no costs, no matchings),
so that the oracle and the GPU library stay independent of each other.

Units handed to both sides: latency in seconds, bandwidth in bytes/second, sizes in bytes, so the
cost 2(alpha + c/beta) of the paper's Eqs. 2-3 comes out in seconds (the unit the paper's
appendix quotes for the estimated cost).

The synthetic networks stand in for the paper's measured AWS scenarios (Sec. 4.1, Cases 1-5, and
the appendix's network-benchmark tables): same shapes (regions x devices per region), same value
ranges (intra-region fast / inter-region slow), generated with numpy's default_rng.
"""
from __future__ import annotations

import os
from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

MS = 1e-3                 # milliseconds -> seconds
GBPS = 1e9 / 8.0          # Gbit/s -> bytes/s

_GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tests", "golden")


@dataclass
class Workload:
    name: str
    N: int
    D_dp: int
    D_pp: int
    c_dp: float
    c_pp: float
    latency: np.ndarray      # N x N, seconds
    bandwidth: np.ndarray    # N x N, bytes / second
    P: int                   # population size the config names
    extra: Dict = field(default_factory=dict)


def _mirror(upper: np.ndarray) -> np.ndarray:
    """Symmetric matrix from the strict upper triangle of `upper`; diagonal set to 1 (unused)."""
    u = np.triu(upper, 1)
    m = u + u.T
    np.fill_diagonal(m, 1.0)
    return m


def network_iid(N: int, seed: int, lat_ms=(1.0, 100.0), log10_bw_gbps=(-1.0, 1.0)):
    """Per-pair iid symmetric network: latency U[lo,hi] ms, bandwidth 10^U[lo,hi] Gbps."""
    rng = np.random.default_rng(seed)
    lat = rng.uniform(lat_ms[0], lat_ms[1], size=(N, N))
    bw = 10.0 ** rng.uniform(log10_bw_gbps[0], log10_bw_gbps[1], size=(N, N))
    return _mirror(lat) * MS, _mirror(bw) * GBPS


def network_regions(n_regions: int, per_region: int, seed: int,
                    intra_bw_gbps=(5.0, 10.0), intra_lat_ms=(0.5, 5.0),
                    inter_bw_gbps=(0.1, 2.0), inter_lat_ms=(20.0, 250.0),
                    jitter=0.05):
    """Geo-distributed network: `n_regions` regions of `per_region` devices (device d lives in
    region d // per_region). One base (latency, bandwidth) value per region pair, symmetric at
    region level, inter-region bandwidth log-uniform; then a per-device-pair multiplicative jitter
    U[1-jitter, 1+jitter] (symmetric) so that device pairs of one region pair do not tie exactly."""
    rng = np.random.default_rng(seed)
    R = n_regions
    N = R * per_region
    base_lat = rng.uniform(inter_lat_ms[0], inter_lat_ms[1], size=(R, R))
    base_bw = 10.0 ** rng.uniform(np.log10(inter_bw_gbps[0]), np.log10(inter_bw_gbps[1]), size=(R, R))
    base_lat = np.triu(base_lat, 1) + np.triu(base_lat, 1).T
    base_bw = np.triu(base_bw, 1) + np.triu(base_bw, 1).T
    np.fill_diagonal(base_lat, rng.uniform(intra_lat_ms[0], intra_lat_ms[1], size=R))
    np.fill_diagonal(base_bw, rng.uniform(intra_bw_gbps[0], intra_bw_gbps[1], size=R))
    region = np.arange(N) // per_region
    lat = base_lat[np.ix_(region, region)]
    bw = base_bw[np.ix_(region, region)]
    if jitter > 0.0:
        jl = rng.uniform(1.0 - jitter, 1.0 + jitter, size=(N, N))
        jb = rng.uniform(1.0 - jitter, 1.0 + jitter, size=(N, N))
        lat = lat * (np.triu(jl, 1) + np.triu(jl, 1).T + np.eye(N))
        bw = bw * (np.triu(jb, 1) + np.triu(jb, 1).T + np.eye(N))
    np.fill_diagonal(lat, 1.0 / MS)
    np.fill_diagonal(bw, 1.0)
    return lat * MS, bw * GBPS


def network_clustered(n_regions: int, per_region: int, n_clusters: int, seed: int, jitter=0.05):
    """Clustered geo network: regions grouped into `n_clusters` clusters. Intra-region
    2-10 Gbps / 0.5-5 ms; same cluster 1.0-1.3 Gbps / 10-70 ms (the paper's regional range,
    Sec. 4.1 Case 4); across clusters 0.3-1.3 Gbps / 70-250 ms (world-wide range, Case 5)."""
    rng = np.random.default_rng(seed)
    R = n_regions
    N = R * per_region
    cl = np.arange(R) // (R // n_clusters)
    same = cl[:, None] == cl[None, :]
    lat_same = rng.uniform(10.0, 70.0, size=(R, R))
    lat_diff = rng.uniform(70.0, 250.0, size=(R, R))
    bw_same = rng.uniform(1.0, 1.3, size=(R, R))
    bw_diff = rng.uniform(0.3, 1.3, size=(R, R))
    base_lat = np.where(same, lat_same, lat_diff)
    base_bw = np.where(same, bw_same, bw_diff)
    base_lat = np.triu(base_lat, 1) + np.triu(base_lat, 1).T
    base_bw = np.triu(base_bw, 1) + np.triu(base_bw, 1).T
    np.fill_diagonal(base_lat, rng.uniform(0.5, 5.0, size=R))
    np.fill_diagonal(base_bw, rng.uniform(2.0, 10.0, size=R))
    region = np.arange(N) // per_region
    lat = base_lat[np.ix_(region, region)]
    bw = base_bw[np.ix_(region, region)]
    jl = rng.uniform(1.0 - jitter, 1.0 + jitter, size=(N, N))
    jb = rng.uniform(1.0 - jitter, 1.0 + jitter, size=(N, N))
    lat = lat * (np.triu(jl, 1) + np.triu(jl, 1).T + np.eye(N))
    bw = bw * (np.triu(jb, 1) + np.triu(jb, 1).T + np.eye(N))
    np.fill_diagonal(lat, 1.0 / MS)
    np.fill_diagonal(bw, 1.0)
    return lat * MS, bw * GBPS


def network_homogeneous(N: int, bw_gbps: float = 100.0, lat_ms: float = 0.1):
    """Every device pair identical (the data-centre case of the paper's Sec. 3 opening)."""
    lat = np.full((N, N), lat_ms * MS)
    bw = np.full((N, N), bw_gbps * GBPS)
    return lat, bw


def _read_region_table(fname: str):
    names, intra_lat, intra_bw, sect = None, None, None, None
    rows = {"delay_ms": [], "bandwidth_gbps": []}
    with open(os.path.join(_GOLDEN, fname)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0] == "regions":
                names = tok[1:]
            elif tok[0] == "intra_delay_ms":
                intra_lat = float(tok[1])
            elif tok[0] == "intra_bandwidth_gbps":
                intra_bw = float(tok[1])
            elif tok[0] in rows:
                sect = tok[0]
            else:
                rows[sect].append([np.nan if t == "-" else float(t) for t in tok])
    lat = np.array(rows["delay_ms"])
    bw = np.array(rows["bandwidth_gbps"])
    np.fill_diagonal(lat, intra_lat)
    np.fill_diagonal(bw, intra_bw)
    return names, lat, bw


def network_paper_table(fname: str, per_region: int):
    """Network built verbatim from one of the paper's printed region tables (text fixture under
    tests/golden/), `per_region` devices per region, no jitter: every device pair of one region
    pair ties exactly."""
    _, lat_r, bw_r = _read_region_table(fname)
    R = lat_r.shape[0]
    region = np.arange(R * per_region) // per_region
    lat = lat_r[np.ix_(region, region)].copy()
    bw = bw_r[np.ix_(region, region)].copy()
    np.fill_diagonal(lat, 1.0 / MS)
    np.fill_diagonal(bw, 1.0)
    return lat * MS, bw * GBPS


def network_two_site_asymmetric(per_site: int):
    """Two-site network with the slightly asymmetric inter-site bandwidth the paper's appendix
    reports for its real deployment (3.87 Gbps one way, 3.73 Gbps the other; 21.8 ms; intra-site
    0.5 ms with 10.40 / 11.98 Gbps). Exercises the symmetrisation of Sec. 2."""
    N = 2 * per_site
    site = np.arange(N) // per_site
    lat = np.where(site[:, None] == site[None, :], 0.5, 21.8)
    bw = np.empty((N, N))
    for a in range(N):
        for b in range(N):
            if site[a] == site[b]:
                bw[a, b] = 10.40 if site[a] == 0 else 11.98
            else:
                bw[a, b] = 3.87 if site[a] == 0 else 3.73
    np.fill_diagonal(lat, 1.0 / MS)
    np.fill_diagonal(bw, 1.0)
    return lat * MS, bw * GBPS


def random_population(P: int, N: int, seed: int) -> np.ndarray:
    """P uniformly random permutations of 0..N-1, int32, row-major P x N."""
    rng = np.random.default_rng(seed)
    out = np.empty((P, N), dtype=np.int32)
    for p in range(P):
        out[p] = rng.permutation(N)
    return out


# GPT-1.3B-shaped message sizes: activations of one micro-batch hop b*s*h*2 bytes (fp16), and
# gradients of one of D_pp stages (1.3e9 parameters * 2 bytes / D_pp).
def gpt13b_sizes(D_pp: int, b: int = 1, s: int = 2048, h: int = 2048) -> Tuple[float, float]:
    c_pp = float(b * s * h * 2)
    c_dp = 1.3e9 * 2.0 / D_pp
    return c_dp, c_pp


def config(name: str) -> Workload:
    """The benchmark configurations, by name: C1..C5, plus C2b (paper Case-5 table verbatim) and
    C3h (homogeneous tie check)."""
    if name == "C1":
        lat, bw = network_iid(8, seed=0)
        return Workload("C1", 8, 2, 4, 25e6, 4e6, lat, bw, 64)
    if name in ("C2", "C3"):
        lat, bw = network_regions(8, 8, seed=0)
        c_dp, c_pp = gpt13b_sizes(8)
        return Workload(name, 64, 8, 8, c_dp, c_pp, lat, bw, 4096,
                        {"ls_rounds": 20} if name == "C3" else {})
    if name == "C2b":
        lat, bw = network_paper_table("paper_case5_network.txt", 8)
        c_dp, c_pp = gpt13b_sizes(8)
        return Workload("C2b", 64, 8, 8, c_dp, c_pp, lat, bw, 4096)
    if name == "C3h":
        lat, bw = network_homogeneous(64)
        c_dp, c_pp = gpt13b_sizes(8)
        return Workload("C3h", 64, 8, 8, c_dp, c_pp, lat, bw, 4096, {"ls_rounds": 20})
    if name == "C4":
        lat, bw = network_regions(16, 16, seed=0, inter_bw_gbps=(0.05, 5.0), inter_lat_ms=(10.0, 250.0))
        c_dp, c_pp = gpt13b_sizes(16)
        return Workload("C4", 256, 16, 16, c_dp, c_pp, lat, bw, 1024)
    if name == "C5":
        lat, bw = network_clustered(32, 32, 4, seed=7)
        c_dp, c_pp = gpt13b_sizes(16)
        return Workload("C5", 1024, 64, 16, c_dp, c_pp, lat, bw, 4096,
                        {"generations": 100, "philox_seed": 7})
    raise KeyError(name)
