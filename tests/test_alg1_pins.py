"""Pins of the Algorithm 1 oracle (oracle/alg1_oracle.c): values worked by hand, invariants and
special cases, none of them produced by the oracle or by the HIP path."""
import os

import numpy as np
import pytest

from paper_2604_00317_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def parallel_links(caps, n_comm=1):
    """n_comm pairs that all have the same candidates: one single-link path per link."""
    m = len(caps)
    cp = np.arange(n_comm + 1, dtype=np.int32) * m
    lp = np.arange(n_comm * m + 1, dtype=np.int32)
    pl = np.tile(np.arange(m, dtype=np.int32), n_comm)
    return (m, np.asarray(caps, dtype=np.float64), n_comm, cp, n_comm * m, lp, pl)


def test_worked_example(oracle_mod):
    line = [l for l in open(os.path.join(GOLDEN, "alg1_worked_example.txt")) if l[0] != "#"][0]
    f0, f1, lam, sweeps = line.split()
    r = oracle_mod.alg1(*parallel_links([100.0, 50.0]), [8.0], 0.5, 1.0)
    assert r["flows"].tolist() == [float(f0), float(f1)]
    assert r["lam"] == float(lam) and r["sweeps"] == int(sweeps)


def test_gauss_seidel_schedule(oracle_mod):
    """Two identical pairs over two equal links, everything routed in one sweep: the second pair
    already sees the first one's load and takes the other link (a Jacobi schedule would put
    both on link 0)."""
    r = oracle_mod.alg1(*parallel_links([10.0, 10.0], n_comm=2), [4.0, 4.0], 1.0, 1.0)
    assert r["flows"].tolist() == [4.0, 0.0, 0.0, 4.0]
    assert r["sweeps"] == 1 and r["lam"] == 0.4


def test_bottleneck_not_additive_cost(oracle_mod):
    """Links e0, e1 carry 3, link e2 carries 5 (capacity 10 each).  The third pair lists [e2]
    before [e0, e1]: the bottleneck costs are 0.5 and max(0.3, 0.3) = 0.3, so it moves to the
    second candidate; an additive cost (0.6) would have kept the first."""
    cp = np.array([0, 1, 2, 4], dtype=np.int32)
    lp = np.array([0, 2, 3, 4, 6], dtype=np.int32)
    pl = np.array([0, 1, 2, 2, 0, 1], dtype=np.int32)
    r = oracle_mod.alg1(3, [10.0, 10.0, 10.0], 3, cp, 4, lp, pl, [3.0, 5.0, 1.0], 1.0, 1.0)
    assert r["flows"].tolist() == [3.0, 5.0, 0.0, 1.0]
    assert r["load"].tolist() == [4.0, 4.0, 5.0]


def test_chunk_multiples_and_residual(oracle_mod):
    """d = 10, phi = 0.5, chi = 4: 4 (floor(5/4) chunks), then r = 6 -> 4 (floor(3/4) = 0 chunks:
    one chunk), then the residual 2 < chi.  Equal links, so the candidates alternate."""
    r = oracle_mod.alg1(*parallel_links([1.0, 1.0]), [10.0], 0.5, 4.0)
    assert r["sweeps"] == 3
    assert r["flows"].tolist() == [6.0, 4.0]        # 4 on link 0, 4 on link 1, 2 on link 0 (tie)


def test_single_chunk_rule_terminates(oracle_mod):
    r = oracle_mod.alg1(*parallel_links([1.0]), [3.0], 0.1, 1.0)
    assert r["sweeps"] == 3 and r["flows"].tolist() == [3.0]


def test_phi_one_routes_everything_at_once(oracle_mod):
    w = W.make_config(0)
    d = np.floor(w.traffic / 4096.0) * 4096.0
    r = oracle_mod.alg1(*w.topo.csr(), d, 1.0, 4096.0)
    assert r["sweeps"] == 1
    # one candidate per pair carries the whole demand
    cp = w.topo.comm_path_ptr
    for k in range(w.topo.n_comm):
        f = r["flows"][cp[k]:cp[k + 1]]
        assert f.max() == d[k] and f.sum() == d[k]


def test_zero_traffic(oracle_mod):
    w = W.make_config(0)
    r = oracle_mod.alg1(*w.topo.csr(), np.zeros(w.topo.n_comm), 0.5, 1.0)
    assert r["sweeps"] == 0 and r["lam"] == 0.0 and not r["flows"].any()


@pytest.mark.parametrize("cfg", [0, 1])
def test_invariants(oracle_mod, cfg):
    """Flows of a pair add up to its demand exactly, every flow is a whole number of chunks up
    to one residual per pair, lambda is the congestion of the returned flows, and splitting
    beats the direct-path-only plan on skewed traffic."""
    w = W.make_config(cfg)
    t = w.topo
    chi = float(1 << 20)
    r = oracle_mod.alg1(*t.csr(), w.traffic, 0.5, chi)
    cp = t.comm_path_ptr
    for k in range(t.n_comm):
        f = r["flows"][cp[k]:cp[k + 1]]
        assert f.sum() == w.traffic[k]
        assert np.count_nonzero(np.mod(f, chi)) <= 1
    load = np.zeros(t.n_links)
    for p in range(t.n_paths):
        load[t.path_links[t.path_link_ptr[p]:t.path_link_ptr[p + 1]]] += r["flows"][p]
    assert np.array_equal(load, r["load"])
    assert r["lam"] == (load / t.cap).max()
    static = np.zeros(t.n_links)
    for k in range(t.n_comm):
        p = cp[k]
        static[t.path_links[t.path_link_ptr[p]:t.path_link_ptr[p + 1]]] += w.traffic[k]
    assert r["lam"] < (static / t.cap).max()


def transcription(csr, demand, phi, chi):
    """The steps of the listing once more, in plain Python, for tiny inputs."""
    n_links, cap, n_comm, cp, n_paths, lp, pl = csr
    L = [0.0] * n_links
    c = [0.0] * n_links
    r = [float(x) for x in demand]
    flows = [0.0] * n_paths
    sweeps = 0
    while any(x > 0 for x in r):
        sweeps += 1
        for k in range(n_comm):
            if r[k] <= 0:
                continue
            best, pb = float("inf"), None
            for p in range(cp[k], cp[k + 1]):
                cost = max([c[e] for e in pl[lp[p]:lp[p + 1]]] + [0.0])
                if cost < best:
                    best, pb = cost, p
            if r[k] < chi:
                f = r[k]
            else:
                f = np.floor(r[k] * phi / chi) * chi
                if f <= 0:
                    f = chi
            flows[pb] += f
            for e in pl[lp[pb]:lp[pb + 1]]:
                L[e] += f
                c[e] = L[e] * (1.0 / cap[e])
            r[k] -= f
    return flows, sweeps


@pytest.mark.parametrize("seed", range(6))
def test_against_transcription_on_tiny_inputs(oracle_mod, seed):
    rng = np.random.default_rng(seed)
    t = W.random_topology(rng, int(rng.integers(3, 12)), int(rng.integers(1, 9)), 5, 3)
    d = rng.integers(0, 200, size=t.n_comm).astype(np.float64)
    phi = float(rng.choice([0.25, 0.5, 0.9, 1.0]))
    chi = float(rng.choice([1.0, 3.0, 16.0]))
    r = oracle_mod.alg1(*t.csr(), d, phi, chi)
    flows, sweeps = transcription(t.csr(), d, phi, chi)
    assert r["flows"].tolist() == flows and r["sweeps"] == sweeps
