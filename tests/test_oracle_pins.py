"""Pins of the CPU oracle against facts it did not produce itself (no GPU needed).

Each test names the mistake it is meant to catch.  Sources: closed forms of the
min-congestion problem (Eq. (1)-(5), Sec. IV-B, capacity-normalized), the paper's stated
theoretical gains (tests/golden/theoretical_speedups.txt), the multiplicative-weights
guarantee lambda <= (1+eps)^2 lambda* for T >= T_min, an exact LP optimum from a brute-force
simplex, and hand-derived trajectories on two-link instances.
"""
import math
import os

import numpy as np
import pytest

from oracle.lp_simplex import min_congestion_lp, simplex_standard
from paper_2604_00317_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def parallel_links(caps):
    m = len(caps)
    return dict(n_links=m, cap=np.asarray(caps, dtype=np.float64), n_comm=1,
                comm_path_ptr=[0, m], n_paths=m, path_link_ptr=list(range(m + 1)),
                path_links=list(range(m)))


def run(oracle_mod, t, demand, eps, iters, **kw):
    if isinstance(t, W.Topology):
        return oracle_mod.solve(*t.csr(), demand, eps, iters, **kw)
    return oracle_mod.solve(t["n_links"], t["cap"], t["n_comm"], t["comm_path_ptr"],
                            t["n_paths"], t["path_link_ptr"], t["path_links"], demand, eps,
                            iters, **kw)


def t_min(rho, lam_star, n_links, eps):
    return math.ceil(rho * math.log(n_links) / (eps * eps * (1 - eps - eps * eps) * lam_star))


# (i) equal parallel links: round robin, exact split, exact lambda ----------------------------
@pytest.mark.parametrize("m,T", [(2, 10), (3, 300), (4, 200), (7, 700)])
def test_equal_parallel_links_round_robin(oracle_mod, m, T):
    cap = 50e9
    d = 3.0e8
    r = run(oracle_mod, parallel_links([cap] * m), [d], 0.1, T)
    assert r["count"].tolist() == [T // m] * m          # catches a wrong tie rule / update
    assert r["lam"] == pytest.approx(d / (m * cap), rel=1e-14)


# (ii) unequal parallel links: lambda* = d / sum(cap) --------------------------------------------
@pytest.mark.parametrize("caps", [[100e9, 50e9, 50e9], [100e9, 25e9], [200e9, 100e9, 50e9, 50e9]])
def test_unequal_parallel_links_within_band(oracle_mod, caps):
    eps, d = 0.1, 1.0e6
    lam_star = d / sum(caps)
    rho = d / min(caps)
    T = t_min(rho, lam_star, len(caps), eps)
    r = run(oracle_mod, parallel_links(caps), [d], eps, T)
    assert lam_star * (1 - 1e-12) <= r["lam"] <= (1 + eps) ** 2 * lam_star
    # a link cannot carry more than its congestion budget: split_i * d / cap_i <= lambda
    for s, c in zip(r["splits"], caps):
        assert s <= (1 + eps) ** 2 * c / sum(caps) + 1e-12
    # a longer run settles near the optimum, within the eps-sized limit cycle of a fixed step
    # (price = len instead of len/cap would give equal thirds: 1.33 lambda* on the first case)
    r2 = run(oracle_mod, parallel_links(caps), [d], eps, 20 * T)
    assert r2["lam"] <= (1 + eps / 2) * lam_star
    np.testing.assert_allclose(r2["splits"], np.asarray(caps) / sum(caps), atol=0.02)


def test_first_switch_iteration_hand_derived(oracle_mod):
    """Two links, caps 100 and 50 GB/s, eps 0.1.  rho = d/50e9, so the fast link's normalised
    load is 1/2 and its length grows by 1.05 per iteration; it stays cheapest while
    1.05^n / 100 <= 1 / 50, i.e. for n <= 14 (1.05^14 = 1.9799, 1.05^15 = 2.0789).  The slow
    link is therefore first chosen in iteration 15 (0-based).  Catches a wrong eps, a missing
    1/rho, price without 1/cap, or `<=` instead of `<`."""
    t = parallel_links([100e9, 50e9])
    assert run(oracle_mod, t, [1e6], 0.1, 15)["count"].tolist() == [15, 0]
    assert run(oracle_mod, t, [1e6], 0.1, 16)["count"].tolist() == [15, 1]
    # after the switch the slow link has normalised load 1: length 1.1, price 1.1/50 = 0.022
    # against 2.0789/100 = 0.0208 -> back to the fast link in iteration 16
    assert run(oracle_mod, t, [1e6], 0.1, 17)["count"].tolist() == [16, 1]


def test_jacobi_schedule_two_commodities(oracle_mod):
    """Two identical commodities over the same two equal links.  Under the Jacobi schedule both
    see the same prices, so both take link 0, then both take link 1, alternating: every
    commodity ends with counts [T/2, T/2] and each iteration loads one link with 2d, giving
    lambda = d / cap.  A Gauss-Seidel sweep would instead pin commodity 0 to link 0."""
    cap, d, T = 50e9, 1.0e6, 100
    r = oracle_mod.solve(2, [cap, cap], 2, [0, 2, 4], 4, [0, 1, 2, 3, 4], [0, 1, 0, 1],
                         [d, d], 0.1, T)
    assert r["count"].tolist() == [T // 2, T // 2, T // 2, T // 2]
    assert r["lam"] == pytest.approx(d / cap, rel=1e-14)


# (iii) balanced traffic keeps the direct path -------------------------------------------------
@pytest.mark.parametrize("G", [4, 8])
def test_uniform_traffic_stays_direct(oracle_mod, G):
    t = W.build_fabric(1, G)
    D, T = float(1 << 23), 120
    r = run(oracle_mod, t, np.full(t.n_comm, D), 0.1, T)
    cp = t.comm_path_ptr
    assert np.all(r["count"][cp[:-1]] == T)
    assert r["count"].sum() == T * t.n_comm
    assert r["lam"] == pytest.approx(D / W.INTRA_CAP, rel=1e-13)


# (vi) one path per commodity: static congestion ------------------------------------------------
def test_single_path_is_static_congestion(oracle_mod):
    rng = np.random.default_rng(5)
    E, K = 9, 20
    cap = rng.choice([25.0, 50.0, 100.0], size=E) * 1e9
    lp, pl = [0], []
    for _ in range(K):
        pl += rng.choice(E, size=int(rng.integers(1, 4)), replace=False).tolist()
        lp.append(len(pl))
    d = np.floor(rng.random(K) * 1e7) + 1
    r = oracle_mod.solve(E, cap, K, list(range(K + 1)), K, lp, pl, d, 0.1, 37)
    load = np.zeros(E)
    for k in range(K):
        for i in range(lp[k], lp[k + 1]):
            load[pl[i]] += d[k]
    assert r["lam"] == pytest.approx((load / cap).max(), rel=1e-13)
    assert np.all(r["splits"] == 1.0)


# (vii) one hot pair: the paper's theoretical gains -------------------------------------------
def _golden_speedups():
    rows = []
    with open(os.path.join(GOLDEN, "theoretical_speedups.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, g, n, r, gain = line.split()
                rows.append((name, int(g), int(n), int(r), float(gain)))
    return rows


@pytest.mark.parametrize("name,G,N,R,gain", _golden_speedups())
def test_single_hot_pair_matches_paper_gain(oracle_mod, name, G, N, R, gain):
    access = [[r] for r in range(R)] if R else None       # 1:1 GPU-NIC affinity (Sec. IV-B)
    t = W.build_fabric(N, G, R, access)
    d = np.zeros(t.n_comm)
    # pair (0 -> 1) inside a node, or GPU 0 of node 0 -> GPU 0 of node 1
    k = 0 if N == 1 else int(np.nonzero((t.src == 0) & (t.dst == G))[0][0])
    d[k] = 1.0e8
    eps = 0.1
    if N == 1:
        single = d[k] / W.INTRA_CAP
    else:
        single = d[k] / W.NIC_CAP
    lam_star = single / gain
    # width: intra -> relay paths put d on 100 GB/s links; inter -> NIC links at 50 GB/s
    rho = single
    T = t_min(rho, lam_star, t.n_links, eps)
    r = run(oracle_mod, t, d, eps, T)
    assert lam_star * (1 - 1e-12) <= r["lam"] <= (1 + eps) ** 2 * lam_star
    r1 = run(oracle_mod, t, d, eps, 1)                  # first choice = the single default path
    assert r1["lam"] == pytest.approx(single, rel=1e-14)


def test_single_hot_pair_mesh8(oracle_mod):
    t = W.build_fabric(1, 8)
    d = np.zeros(t.n_comm)
    d[3] = 7.0e8
    lam_star = d[3] / (7 * W.INTRA_CAP)
    cp = t.comm_path_ptr
    # bottleneck cost: 7 link-disjoint paths of equal capacity tie whenever their lengths are
    # equal, so the candidates are taken in exact round robin
    r = run(oracle_mod, t, d, 0.1, 700, flags=1)
    assert r["count"][cp[3]:cp[4]].tolist() == [100] * 7
    assert r["lam"] == pytest.approx(lam_star, rel=1e-13)
    # sum cost: a relay path pays for two links, so the direct link is favoured, but the
    # result stays inside the guarantee (width rho = d/cap = 7 lambda*)
    T = t_min(7 * lam_star, lam_star, t.n_links, 0.1)
    r = run(oracle_mod, t, d, 0.1, T)
    assert lam_star * (1 - 1e-12) <= r["lam"] <= 1.21 * lam_star
    assert r["count"][cp[3]] > r["count"][cp[3] + 1]


# (iv) exact LP optimum on tiny inputs ------------------------------------------------------------
def test_simplex_against_scipy():
    from scipy.optimize import linprog
    rng = np.random.default_rng(11)
    for _ in range(5):
        m, n = 4, 9
        A = rng.random((m, n))
        x0 = rng.random(n)
        b = A @ x0
        c = rng.random(n)
        obj, x = simplex_standard(c, A, b)
        ref = linprog(c, A_eq=A, b_eq=b, bounds=(0, None), method="highs")
        assert obj == pytest.approx(ref.fun, rel=1e-8, abs=1e-10)
        assert np.allclose(A @ x, b, atol=1e-8) and np.all(x >= -1e-9)


@pytest.mark.parametrize("G,seed", [(4, 0), (4, 1), (5, 2), (5, 3)])
def test_lambda_within_band_of_lp_optimum(oracle_mod, G, seed):
    t = W.build_fabric(1, G)
    rng = np.random.default_rng(seed)
    d = np.floor(rng.pareto(1.2, t.n_comm) * 1e6) + 1.0
    lam_star, x_star = min_congestion_lp(t.n_links, t.cap, t.comm_path_ptr, t.path_link_ptr,
                                         t.path_links, d)
    # the simplex answer is feasible and reproduces its own objective
    lam_chk, _ = oracle_mod.congestion(t.n_links, t.cap, t.comm_path_ptr, t.path_link_ptr,
                                       t.path_links, d, x_star)
    assert lam_chk == pytest.approx(lam_star, rel=1e-9)
    eps = 0.1
    # width as the method defines it: demand that can reach a link, over its capacity
    reach = np.zeros(t.n_links)
    for k in range(t.n_comm):
        links = set()
        for p in range(t.comm_path_ptr[k], t.comm_path_ptr[k + 1]):
            links.update(t.path_links[t.path_link_ptr[p]:t.path_link_ptr[p + 1]].tolist())
        for e in links:
            reach[e] += d[k]
    rho = (reach / t.cap).max()
    T = t_min(rho, lam_star, t.n_links, eps)
    r = run(oracle_mod, t, d, eps, T, want_lb=True)
    assert lam_star * (1 - 1e-9) <= r["lam"] <= (1 + eps) ** 2 * lam_star
    assert r["lb"].max() <= lam_star * (1 + 1e-9)          # weak duality
    assert r["lb"].max() >= lam_star / (1 + eps) ** 2        # and it is tight


def test_lp_optimum_inter_node_tiny(oracle_mod):
    t = W.build_fabric(2, 2, 2, [[0], [1]])
    rng = np.random.default_rng(4)
    d = np.floor(rng.pareto(1.0, t.n_comm) * 1e6) + 1.0
    lam_star, _ = min_congestion_lp(t.n_links, t.cap, t.comm_path_ptr, t.path_link_ptr,
                                    t.path_links, d)
    r = run(oracle_mod, t, d, 0.1, 6000, want_lb=True)
    assert lam_star * (1 - 1e-9) <= r["lam"] <= 1.21 * lam_star
    assert r["lb"].max() <= lam_star * (1 + 1e-9)


# (v) invariants on the benchmark shapes ------------------------------------------------------
@pytest.mark.parametrize("cfg", [0, 1, 3])
def test_invariants_on_configs(oracle_mod, cfg):
    w = W.make_config(cfg)
    t = w.topo
    iters = w.iters if cfg < 3 else 120
    r = run(oracle_mod, t, w.traffic, w.eps, iters, want_lb=True)
    per_comm = np.add.reduceat(r["count"].astype(np.int64), t.comm_path_ptr[:-1])
    assert np.all(per_comm == iters)
    np.testing.assert_allclose(np.add.reduceat(r["splits"], t.comm_path_ptr[:-1]), 1.0,
                               rtol=0, atol=1e-12)
    lam2, util = oracle_mod.congestion(t.n_links, t.cap, t.comm_path_ptr, t.path_link_ptr,
                                       t.path_links, w.traffic, r["splits"])
    assert r["lam"] == pytest.approx(lam2, rel=1e-11)       # linearity of the congestion
    np.testing.assert_allclose(r["sumload"] / iters, util, rtol=1e-10, atol=0)
    assert r["lb"].max() <= r["lam"] * (1 + 1e-12)
    # endpoint cut bounds: all egress of a GPU must cross its outgoing links (GPU links and
    # GPU->NIC links), likewise ingress
    G, N = t.meta["gpus_per_node"], t.meta["n_nodes"]
    m = len(t.meta["access"][0]) if t.meta["rails"] else 0
    nic_out = np.zeros(G)
    for acc in t.meta["access"]:
        for g in acc:
            nic_out[g] += W.NIC_CAP
    for g in range(N * G):
        out_cap = (G - 1) * W.INTRA_CAP + nic_out[g % G]
        assert r["lam"] >= w.traffic[t.src == g].sum() / out_cap * (1 - 1e-12)
        assert r["lam"] >= w.traffic[t.dst == g].sum() / out_cap * (1 - 1e-12)


# (viii) metamorphic -----------------------------------------------------------------------------
def test_power_of_two_scaling_and_relabelling(oracle_mod):
    w = W.make_config(1)
    t = w.topo
    base = run(oracle_mod, t, w.traffic, w.eps, 150)
    r = run(oracle_mod, t, w.traffic * 8.0, w.eps, 150)
    assert np.array_equal(r["count"], base["count"]) and r["lam"] == base["lam"] * 8.0
    t2 = W.Topology(**{**t.__dict__, "cap": t.cap * 4.0})
    r = run(oracle_mod, t2, w.traffic, w.eps, 150)
    assert np.array_equal(r["count"], base["count"]) and r["lam"] == base["lam"] / 4.0
    perm = np.random.default_rng(3).permutation(t.n_links)      # new id of old link e
    cap3 = np.empty_like(t.cap)
    cap3[perm] = t.cap
    t3 = W.Topology(**{**t.__dict__, "cap": cap3,
                       "path_links": perm[t.path_links].astype(np.int32)})
    r = run(oracle_mod, t3, w.traffic, w.eps, 150)
    assert np.array_equal(r["count"], base["count"]) and r["lam"] == base["lam"]


def test_zero_traffic_and_zero_demand_commodities(oracle_mod):
    t = W.build_fabric(1, 4)
    r = run(oracle_mod, t, np.zeros(t.n_comm), 0.1, 10)
    assert r["lam"] == 0.0
    assert np.all(r["count"][t.comm_path_ptr[:-1]] == 10)
    d = np.zeros(t.n_comm)
    d[0] = 5e6
    r = run(oracle_mod, t, d, 0.1, 30)
    assert np.all(np.add.reduceat(r["count"], t.comm_path_ptr[:-1]) == 30)


def test_bottleneck_cost_mode(oracle_mod):
    """Max-of-links path cost (the paper's choice, Sec. IV-B).  With equal initial lengths
    every candidate ties, so iteration 0 takes the direct path; one hot pair on a 4-GPU mesh
    then rotates over its 3 link-disjoint paths exactly."""
    t = W.build_fabric(1, 4)
    d = np.zeros(t.n_comm)
    d[0] = 3.0e8
    r = run(oracle_mod, t, d, 0.1, 300, flags=1)
    assert r["count"][:3].tolist() == [100, 100, 100]
    assert r["lam"] == pytest.approx(d[0] / (3 * W.INTRA_CAP), rel=1e-13)
    r = run(oracle_mod, t, np.full(t.n_comm, 1e6), 0.1, 50, flags=1)
    assert np.all(r["count"][t.comm_path_ptr[:-1]] == 50)


def _golden_line(name, key):
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.split() and line.split()[0] == key:
                return line.split()[1:]
    raise KeyError(key)


def test_bottleneck_price_is_the_length_alone_hand_derived(oracle_mod):
    """Bottleneck mode on two parallel links of unequal capacity (100 and 50 GB/s): the price
    of a link is its length, not length / capacity, so both candidates start level and the
    choices follow tests/golden/bottleneck_two_links.txt (worked by hand from Sec. IV-B's
    bottleneck path cost).  With price = len / cap the faster link would be kept for the first
    15 iterations; equal-capacity pins cannot tell the two apart."""
    want = [int(x) for x in _golden_line("bottleneck_two_links.txt", "fixed")]
    t = parallel_links([100e9, 50e9])
    for T in range(1, len(want) + 1):
        ones = sum(want[:T])
        assert run(oracle_mod, t, [1e6], 0.1, T, flags=1)["count"].tolist() == [T - ones, ones]
    # capacities swapped: the initial prices are lengths too, so the first tie still goes to
    # candidate 0 (initial prices 1/cap would start on the faster link)
    swapped = [int(x) for x in _golden_line("bottleneck_two_links.txt", "fixed_swapped")]
    t2 = parallel_links([50e9, 100e9])
    for T in range(1, len(swapped) + 1):
        ones = sum(swapped[:T])
        assert run(oracle_mod, t2, [1e6], 0.1, T, flags=1)["count"].tolist() == [T - ones, ones]
    # the lengths themselves after the 13 iterations: 1.05^8 and 1.1^5
    r = oracle_mod.solve(2, [100e9, 50e9], 1, [0, 2], 2, [0, 1, 2], [0, 1], [1e6], 0.1, len(want),
                         flags=1, len0=np.ones(2))
    assert r["len"] == pytest.approx([1.05 ** 8, 1.1 ** 5], rel=1e-13)
    # warm start in bottleneck mode prices the given lengths as they are: from (2, 1) link 1
    # is taken until 1.1^n exceeds 2 (n = 8), whatever the capacities
    r = oracle_mod.solve(2, [100e9, 50e9], 1, [0, 2], 2, [0, 1, 2], [0, 1], [1e6], 0.1, 9,
                         flags=1, len0=np.array([2.0, 1.0]))
    assert r["count"].tolist() == [1, 8]


def test_thread_count_does_not_change_results(oracle_mod):
    w = W.make_config(1)
    oracle_mod.set_threads(1)
    a = run(oracle_mod, w.topo, w.traffic, w.eps, 100)
    oracle_mod.set_threads(oracle_mod.max_threads() if oracle_mod.max_threads() > 1 else 4)
    oracle_mod.set_threads(4)
    b = run(oracle_mod, w.topo, w.traffic, w.eps, 100)
    assert np.array_equal(a["count"], b["count"]) and a["lam"] == b["lam"]


def test_width_counts_a_commodity_once_per_link(oracle_mod):
    """One commodity, two candidates sharing their first link: [0,1] and [0,2], caps 50/100/50
    GB/s.  The shared link can be reached by d once, not twice, so rho = d/50e9, link 1's
    normalised load is 1/2 and the trajectory is that of the two-link case: the second
    candidate is first taken in iteration 15.  Counting the commodity once per *path* would
    double rho and delay the switch to iteration 29."""
    r = oracle_mod.solve(3, [50e9, 100e9, 50e9], 1, [0, 2], 2, [0, 2, 4], [0, 1, 0, 2], [1e6],
                         0.1, 16)
    assert r["count"].tolist() == [15, 1]
    assert r["lam"] == pytest.approx(1e6 / 50e9, rel=1e-14)      # the shared link carries all


# ---- warm start (the hysteresis policy read as: start from the previous solve's lengths) ----

def test_warm_start_continues_the_trajectory(oracle_mod):
    """The link lengths are the whole state of the method: T1 iterations followed by T2
    iterations started from the lengths the first run ended with must make exactly the choices
    of one uninterrupted run of T1 + T2 iterations (counts add up, final lengths agree)."""
    for cfg, flags in ((1, 0), (1, 1), (0, 0)):
        w = W.make_config(cfg)
        t = w.topo
        ones = np.ones(t.n_links)
        full = oracle_mod.solve(*t.csr(), w.traffic, w.eps, 50, flags=flags, len0=ones)
        a = oracle_mod.solve(*t.csr(), w.traffic, w.eps, 20, flags=flags, len0=ones)
        b = oracle_mod.solve(*t.csr(), w.traffic, w.eps, 30, flags=flags, len0=a["len"])
        assert np.array_equal(full["count"], a["count"] + b["count"])
        assert np.array_equal(full["len"], b["len"])
        # S restarts at 0 in the second run, so the sums agree up to the rounding of one add
        assert np.allclose(full["sumload"], a["sumload"] + b["sumload"], rtol=1e-14, atol=0)


def test_unit_lengths_are_the_cold_start(oracle_mod):
    w = W.make_config(1)
    t = w.topo
    cold = oracle_mod.solve(*t.csr(), w.traffic, w.eps, 40)
    warm = oracle_mod.solve(*t.csr(), w.traffic, w.eps, 40, len0=np.ones(t.n_links))
    assert np.array_equal(cold["count"], warm["count"]) and cold["lam"] == warm["lam"]


def test_lengths_scaled_by_a_power_of_two_change_nothing(oracle_mod):
    """Only price ratios matter to the argmin; a power of two scales every price exactly."""
    w = W.make_config(1)
    t = w.topo
    a = oracle_mod.solve(*t.csr(), w.traffic, w.eps, 25, len0=np.ones(t.n_links))
    b = oracle_mod.solve(*t.csr(), w.traffic, w.eps, 30, len0=a["len"])
    c = oracle_mod.solve(*t.csr(), w.traffic, w.eps, 30, len0=a["len"] * 0.125)
    assert np.array_equal(b["count"], c["count"]) and b["lam"] == c["lam"]
    assert np.array_equal(b["len"] * 0.125, c["len"])


def test_warm_start_on_new_traffic_keeps_the_loaded_links_expensive(oracle_mod):
    """After a solve for a hot pair the hot pair's direct link is the longest one; a new
    solve for uniform traffic started from those lengths moves traffic off that link in its
    first iteration, which a cold start (everything direct) does not."""
    t = W.build_fabric(1, 8, 0)
    hot = np.zeros(t.n_comm)
    hot[0] = 1e9
    first = oracle_mod.solve(*t.csr(), hot, 0.1, 30, len0=np.ones(t.n_links))
    direct0 = t.path_links[t.path_link_ptr[t.comm_path_ptr[0]]]
    assert first["len"][direct0] == first["len"].max()
    uni = np.full(t.n_comm, 1e6)
    cold = oracle_mod.solve(*t.csr(), uni, 0.1, 1)
    warm = oracle_mod.solve(*t.csr(), uni, 0.1, 1, len0=first["len"])
    assert cold["count"][t.comm_path_ptr[0]] == 1          # direct
    assert warm["count"][t.comm_path_ptr[0]] == 0          # moved to a relay
