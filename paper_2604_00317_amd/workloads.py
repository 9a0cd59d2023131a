"""Seeded synthetic inputs: modeled fabrics (links, capacities, candidate paths as CSR) and
skewed All-to-Allv demand vectors.

This module holds no planner arithmetic.  It only produces the *inputs* that both the HIP
library and the CPU oracle consume, so the two sides can be compared on identical data.

Fabric model (paper Sec. IV-B, "Hop-Adaptive MCF load balancing"): inside a node every GPU pair
has a direct link and may relay through one third GPU of the same node; between nodes only
rail-matched NIC pairs are used, optionally reached through one relay GPU on either side.
Candidate paths are listed in the scan order of Algorithm 1 (direct, then relays ascending,
then NIC paths by rail), which makes "lowest path index" the same tie rule as the strict `<`
scan of that algorithm.

Traffic model: the paper's workloads are synthetic (hot-spot ratio sweep in Sec. V-C, MoE token
counts in Sec. V-D); the generators here produce demands of the same kind -- heavy-tailed
per-destination byte counts -- at the sizes the benchmark configurations name.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

GB = 1.0e9
INTRA_CAP = 100.0 * GB       # directed GPU->GPU link, bytes/s
NIC_CAP = 50.0 * GB          # GPU->NIC, NIC->GPU and NIC->NIC (same rail), bytes/s


@dataclass
class Topology:
    """A modeled fabric in the layout the C ABI takes (all index arrays int32, C order)."""
    n_links: int
    cap: np.ndarray              # float64 [n_links], bytes/s
    n_comm: int
    comm_path_ptr: np.ndarray    # int32 [n_comm+1]
    n_paths: int
    path_link_ptr: np.ndarray    # int32 [n_paths+1]
    path_links: np.ndarray       # int32 [nnz]
    src: np.ndarray              # int32 [n_comm] global GPU id of the source
    dst: np.ndarray              # int32 [n_comm] global GPU id of the destination
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.path_links.shape[0])

    def csr(self):
        return (self.n_links, self.cap, self.n_comm, self.comm_path_ptr, self.n_paths,
                self.path_link_ptr, self.path_links)


def _relay_table(G: int) -> np.ndarray:
    """relay[s, d, j] = j-th local GPU id (ascending) that is neither s nor d."""
    tab = np.zeros((G, G, max(G - 2, 0)), dtype=np.int64)
    for s in range(G):
        for d in range(G):
            if s == d:
                continue
            tab[s, d, :] = [i for i in range(G) if i != s and i != d]
    return tab


def build_fabric(n_nodes: int, gpus_per_node: int = 8, rails: int = 0,
                 access: Optional[Sequence[Sequence[int]]] = None,
                 intra_cap: float = INTRA_CAP, nic_cap: float = NIC_CAP) -> Topology:
    """Links, capacities and candidate paths of `n_nodes` identical nodes.

    access[r] lists the local GPUs that can reach NIC r (all lists the same length m).
    Link id order: intra-node (node, a->b); GPU->NIC (node, rail, GPU in access order);
    NIC->GPU likewise; NIC->NIC (src node, dst node, rail).
    Commodities are all ordered GPU pairs s != d in row-major order of global GPU ids.
    Intra-node candidates: direct, then one relay GPU (ascending).  Inter-node candidates:
    for rail r, for o_s in access[r], for o_d in access[r]:
    [s->o_s if o_s != s], o_s->NIC_r, NIC_r(node)->NIC_r(node'), NIC_r->o_d, [o_d->d if o_d != d].
    """
    N, G, R = int(n_nodes), int(gpus_per_node), int(rails)
    if N < 1 or G < 2:
        raise ValueError("need at least one node with two GPUs")
    if N > 1 and R < 1:
        raise ValueError("more than one node needs at least one rail")
    if N == 1:
        R = 0
    if R > 0:
        acc = np.asarray(access, dtype=np.int64)
        if acc.ndim != 2 or acc.shape[0] != R:
            raise ValueError("access must be [rails][m]")
        m = acc.shape[1]
    else:
        acc = np.zeros((0, 1), dtype=np.int64)
        m = 1

    n_intra = N * G * (G - 1)
    l_acc = R * m                          # GPU->NIC links per node
    base_g2n = n_intra
    base_n2g = base_g2n + N * l_acc
    base_n2n = base_n2g + N * l_acc
    n_n2n = N * (N - 1) * R
    E = base_n2n + n_n2n
    cap = np.empty(E, dtype=np.float64)
    cap[:n_intra] = intra_cap
    cap[n_intra:] = nic_cap

    def intra(node, a, b):
        return node * (G * (G - 1)) + a * (G - 1) + (b - (b > a))

    NG = N * G
    K = NG * (NG - 1)
    s_glob = np.repeat(np.arange(NG, dtype=np.int64), NG - 1)
    off = np.tile(np.arange(NG - 1, dtype=np.int64), NG)
    d_glob = off + (off >= s_glob)
    ns, ls = s_glob // G, s_glob % G
    nd, ld = d_glob // G, d_glob % G
    is_intra = ns == nd

    n_inter_paths = R * m * m
    pmax = max(G - 1, n_inter_paths)
    links = np.full((K, pmax, 5), -1, dtype=np.int32)

    # intra-node commodities: direct + relays
    ki = np.nonzero(is_intra)[0]
    if ki.size:
        links[ki, 0, 0] = intra(ns[ki], ls[ki], ld[ki])
        rt = _relay_table(G)
        for j in range(G - 2):
            rel = rt[ls[ki], ld[ki], j]
            links[ki, 1 + j, 0] = intra(ns[ki], ls[ki], rel)
            links[ki, 1 + j, 1] = intra(ns[ki], rel, ld[ki])

    # inter-node commodities: rail-matched NIC paths with optional relay on each side
    kx = np.nonzero(~is_intra)[0]
    if kx.size:
        nsx, lsx, ndx, ldx = ns[kx], ls[kx], nd[kx], ld[kx]
        pair = nsx * (N - 1) + (ndx - (ndx > nsx))
        j = 0
        for r in range(R):
            for a in range(m):
                o_s = int(acc[r, a])
                for b in range(m):
                    o_d = int(acc[r, b])
                    first = np.where(lsx != o_s, intra(nsx, lsx, o_s), -1)
                    last = np.where(ldx != o_d, intra(ndx, o_d, ldx), -1)
                    links[kx, j, 0] = first
                    links[kx, j, 1] = base_g2n + nsx * l_acc + r * m + a
                    links[kx, j, 2] = base_n2n + pair * R + r
                    links[kx, j, 3] = base_n2g + ndx * l_acc + r * m + b
                    links[kx, j, 4] = last
                    j += 1

    mask = links >= 0
    path_len = mask.sum(axis=2)                      # [K, pmax]
    path_valid = path_len > 0
    npaths = path_valid.sum(axis=1)
    comm_path_ptr = np.zeros(K + 1, dtype=np.int64)
    np.cumsum(npaths, out=comm_path_ptr[1:])
    P = int(comm_path_ptr[-1])
    lens = path_len[path_valid]
    path_link_ptr = np.zeros(P + 1, dtype=np.int64)
    np.cumsum(lens, out=path_link_ptr[1:])
    path_links = links[mask]
    assert path_links.shape[0] == path_link_ptr[-1] < 2 ** 31

    return Topology(
        n_links=int(E), cap=cap, n_comm=int(K),
        comm_path_ptr=comm_path_ptr.astype(np.int32), n_paths=P,
        path_link_ptr=path_link_ptr.astype(np.int32),
        path_links=np.ascontiguousarray(path_links, dtype=np.int32),
        src=s_glob.astype(np.int32), dst=d_glob.astype(np.int32),
        meta=dict(n_nodes=N, gpus_per_node=G, rails=R, access=acc.tolist() if R else [],
                  intra_cap=intra_cap, nic_cap=nic_cap))


def pair_access(rails: int) -> list:
    """GPU pairs {2r, 2r+1} share rail r (4 rails on an 8-GPU node)."""
    return [[2 * r, 2 * r + 1] for r in range(rails)]


def xor_access(rails: int) -> list:
    """One NIC per GPU, each also reachable from the GPU behind the same switch: {r, r^1}."""
    return [sorted((r, r ^ 1)) for r in range(rails)]


# --------------------------------------------------------------------------------------
# traffic
# --------------------------------------------------------------------------------------

def zipf_node_traffic(topo: Topology, seed: int, total_bytes: int = 1 << 26,
                      s: float = 1.2) -> np.ndarray:
    """Per source GPU, `total_bytes` split over the other GPUs by Zipf(s) through a seeded
    permutation; integer byte counts, remainder given to the most popular destination."""
    NG = topo.meta["n_nodes"] * topo.meta["gpus_per_node"]
    rng = np.random.default_rng(seed)
    w = np.arange(1, NG, dtype=np.float64) ** (-s)
    w /= w.sum()
    base = np.floor(total_bytes * w).astype(np.int64)
    base[0] += total_bytes - base.sum()
    d = np.zeros(topo.n_comm, dtype=np.float64)
    for src in range(NG):
        perm = rng.permutation(NG - 1)
        d[src * (NG - 1) + perm] = base
    return d


def hotspot_traffic(topo: Topology, hot_ratio: float, total_bytes: int = 1 << 26,
                    hot_gpu: int = 0) -> np.ndarray:
    """Hot-spot All-to-Allv: every source sends `hot_ratio` of its bytes to one hot GPU and
    spreads the rest evenly (the skew knob of the paper's All-to-Allv sweep)."""
    NG = topo.meta["n_nodes"] * topo.meta["gpus_per_node"]
    d = np.zeros(topo.n_comm, dtype=np.float64)
    for k in range(topo.n_comm):
        s_, t_ = int(topo.src[k]), int(topo.dst[k])
        if s_ == hot_gpu:
            d[k] = total_bytes // (NG - 1)
        elif t_ == hot_gpu:
            d[k] = int(total_bytes * hot_ratio)
        else:
            d[k] = int(total_bytes * (1.0 - hot_ratio)) // max(NG - 2, 1)
    return d


def _inclusion_probabilities(w: np.ndarray, k: int) -> np.ndarray:
    """pi_x = min(1, c*w_x) with sum(pi) = k (water-filling); needs k <= len(w)."""
    w = np.asarray(w, dtype=np.float64)
    order = np.argsort(-w)
    ws = w[order]
    pi = np.zeros_like(ws)
    capped = 0
    while True:
        rest = ws[capped:]
        c = (k - capped) / rest.sum()
        if capped < len(ws) and c * ws[capped] > 1.0:
            capped += 1
            continue
        pi[:capped] = 1.0
        pi[capped:] = c * rest
        break
    out = np.empty_like(pi)
    out[order] = pi
    return out


def moe_traffic(topo: Topology, seed: int, tokens: int, hidden: int, top_k: int,
                n_experts: int, s: float, bytes_per_elem: int = 2,
                rng: Optional[np.random.Generator] = None) -> np.ndarray:
    """MoE dispatch bytes: experts are laid out contiguously over the GPUs, popularity is
    Zipf(s) through a seeded permutation, each source GPU routes tokens*top_k expert slots by a
    multinomial draw over the top-k inclusion probabilities; the local share is dropped."""
    NG = topo.meta["n_nodes"] * topo.meta["gpus_per_node"]
    if n_experts % NG:
        raise ValueError("experts must divide evenly over GPUs")
    per_gpu = n_experts // NG
    if rng is None:
        rng = np.random.default_rng(seed)
    ranks = rng.permutation(n_experts) + 1
    w = ranks.astype(np.float64) ** (-s)
    pi = _inclusion_probabilities(w, top_k)
    pvals = pi / pi.sum()
    d = np.zeros(topo.n_comm, dtype=np.float64)
    for src in range(NG):
        cnt = rng.multinomial(tokens * top_k, pvals)
        per_dst = cnt.reshape(NG, per_gpu).sum(axis=1).astype(np.int64)
        bytes_dst = per_dst * (hidden * bytes_per_elem)
        row = np.delete(bytes_dst, src)
        d[src * (NG - 1):(src + 1) * (NG - 1)] = row
    return d


# --------------------------------------------------------------------------------------
# the benchmark configurations
# --------------------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    topo: Topology
    traffic: np.ndarray          # float64 [n_comm] or [batch, n_comm]
    eps: float
    iters: int
    batch: int = 0               # 0: single plan


CONFIG_NAMES = ["node8_zipf", "2x8_moe_top2", "batch4096_node8_moe", "16x8_moe_top8",
                "64x8_moe_top8"]


def config_topology(i: int) -> Topology:
    if i in (0, 2):
        return build_fabric(1, 8)
    if i == 1:
        return build_fabric(2, 8, 4, pair_access(4))
    if i == 3:
        return build_fabric(16, 8, 4, pair_access(4))
    if i == 4:
        return build_fabric(64, 8, 8, xor_access(8))
    raise ValueError("config index 0..4")


def batch_traffic(topo: Topology, batch: int, first: int = 0) -> np.ndarray:
    """Traffic of the batched configuration: problem b has its own seed and its own skew."""
    out = np.empty((batch, topo.n_comm), dtype=np.float64)
    for b in range(batch):
        rng = np.random.default_rng(2_000_000 + first + b)
        s_b = 0.8 + 0.8 * rng.random()
        out[b] = moe_traffic(topo, 0, tokens=8192, hidden=7168, top_k=2, n_experts=64,
                             s=s_b, rng=rng)
    return out


def make_config(i: int, batch: Optional[int] = None, topo: Optional[Topology] = None) -> Workload:
    """Benchmark configuration i (0..4) with its seeded traffic."""
    if topo is None:
        topo = config_topology(i)
    seed = 1000 + i
    if i == 0:
        return Workload(CONFIG_NAMES[0], topo, zipf_node_traffic(topo, seed), 0.1, 200)
    if i == 1:
        t = moe_traffic(topo, seed, tokens=4096, hidden=4096, top_k=2, n_experts=64, s=1.2)
        return Workload(CONFIG_NAMES[1], topo, t, 0.1, 300)
    if i == 2:
        b = 4096 if batch is None else int(batch)
        return Workload(CONFIG_NAMES[2], topo, batch_traffic(topo, b), 0.1, 200, batch=b)
    if i == 3:
        t = moe_traffic(topo, seed, tokens=8192, hidden=7168, top_k=8, n_experts=256, s=1.4)
        return Workload(CONFIG_NAMES[3], topo, t, 0.05, 1000)
    if i == 4:
        t = moe_traffic(topo, seed, tokens=16384, hidden=7168, top_k=8, n_experts=1024, s=1.6)
        return Workload(CONFIG_NAMES[4], topo, t, 0.05, 1000)
    raise ValueError("config index 0..4")


def random_topology(rng: np.random.Generator, n_links: int, n_comm: int, max_paths: int,
                    max_len: int) -> Topology:
    """An unstructured random instance (ragged path counts and lengths) for parity tests."""
    cap = rng.choice([25.0, 50.0, 100.0, 200.0], size=n_links) * GB
    cp = [0]
    lp = [0]
    pl = []
    for _ in range(n_comm):
        npth = int(rng.integers(1, max_paths + 1))
        for _ in range(npth):
            ln = int(rng.integers(1, min(max_len, n_links) + 1))
            pl.extend(rng.choice(n_links, size=ln, replace=False).tolist())
            lp.append(len(pl))
        cp.append(len(lp) - 1)
    K = n_comm
    return Topology(n_links=n_links, cap=cap.astype(np.float64), n_comm=K,
                    comm_path_ptr=np.asarray(cp, dtype=np.int32), n_paths=len(lp) - 1,
                    path_link_ptr=np.asarray(lp, dtype=np.int32),
                    path_links=np.asarray(pl, dtype=np.int32),
                    src=np.zeros(K, dtype=np.int32), dst=np.zeros(K, dtype=np.int32),
                    meta=dict(kind="random"))


def two_candidate_mesh(G: int) -> Topology:
    """Full mesh of G GPUs (G odd), every ordered pair (s, d) with two candidates: the direct
    link and the relay r = 2d - s mod G, which is neither s nor d and puts exactly one relay
    path on each hop of every link.  K = E = G (G - 1), three pairs per link: small enough for
    the register kernel of the resident regime in every respect but the number of commodities
    and links."""
    assert G % 2 == 1
    link = {}
    for a in range(G):
        for b in range(G):
            if a != b:
                link[(a, b)] = len(link)
    cp, lp, pl = [0], [0], []
    for s in range(G):
        for d in range(G):
            if s == d:
                continue
            r = (2 * d - s) % G
            pl += [link[(s, d)]]
            lp.append(len(pl))
            pl += [link[(s, r)], link[(r, d)]]
            lp.append(len(pl))
            cp.append(len(lp) - 1)
    n = len(link)
    return Topology(n_links=n, cap=np.full(n, 100e9), n_comm=n,
                      comm_path_ptr=np.asarray(cp, dtype=np.int32), n_paths=len(lp) - 1,
                      path_link_ptr=np.asarray(lp, dtype=np.int32),
                      path_links=np.asarray(pl, dtype=np.int32),
                      src=np.zeros(n, dtype=np.int32), dst=np.zeros(n, dtype=np.int32),
                      meta=dict(kind="mesh2"))
