"""Pins of the plan post-processing oracle (oracle/quantize_oracle.py): hand-worked cases and
the properties largest-remainder apportionment is known for."""
import os

import numpy as np
import pytest

from paper_2604_00317_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_worked_examples(oracle_mod):
    for line in open(os.path.join(GOLDEN, "quantize_worked_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, counts, flows = [x.split() for x in line.split("|")]
        d, chi, T = float(head[0]), int(head[1]), int(head[2])
        c = np.array(counts, dtype=np.float64)
        got = oracle_mod.quantize([0, len(c)], [d], c / T, T, chi, 0.0)
        assert got.tolist() == [float(x) for x in flows]


@pytest.mark.parametrize("cfg,chi", [(0, 1 << 20), (1, 65536), (1, 1), (3, 1 << 20)])
def test_apportionment_properties(oracle_mod, cfg, chi):
    w = W.make_config(cfg)
    t = w.topo
    iters = 64
    plan = oracle_mod.solve(*t.csr(), w.traffic, w.eps, iters)
    theta = float(1 << 20)
    flows = oracle_mod.quantize(t.comm_path_ptr, w.traffic, plan["splits"], iters, chi, theta)
    cp = t.comm_path_ptr
    for k in range(t.n_comm):
        f = flows[cp[k]:cp[k + 1]]
        d = w.traffic[k]
        assert f.sum() == d                                   # nothing lost, nothing added
        if d <= theta:                                        # small messages stay direct
            assert f[0] == d and not f[1:].any()
            continue
        c = plan["count"][cp[k]:cp[k + 1]].astype(np.int64)
        N = int(d // chi)
        res = d - N * chi
        jmax = int(np.argmax(c))                              # first of the largest
        whole = f.copy()
        whole[jmax] -= res
        assert not np.mod(whole, chi).any()                   # whole chunks
        chunks = (whole / chi).astype(np.int64)
        lo = (N * c) // iters
        assert ((chunks == lo) | (chunks == lo + 1)).all()    # quota property
        assert chunks.sum() == N
        # a candidate never used gets nothing
        assert not f[c == 0].any()


def test_exact_when_counts_divide(oracle_mod):
    """chi = 1 and T | d: the flows are exactly d * c_j / T."""
    c = np.array([3, 0, 5, 8], dtype=np.float64)
    f = oracle_mod.quantize([0, 4], [1600.0], c / 16, 16, 1, 0.0)
    assert f.tolist() == [300.0, 0.0, 500.0, 800.0]


def test_pairs_are_independent(oracle_mod):
    w = W.make_config(1)
    t = w.topo
    plan = oracle_mod.solve(*t.csr(), w.traffic, w.eps, 50)
    a = oracle_mod.quantize(t.comm_path_ptr, w.traffic, plan["splits"], 50, 4096, 0.0)
    d2 = w.traffic.copy()
    d2[1::2] = 0.0
    b = oracle_mod.quantize(t.comm_path_ptr, d2, plan["splits"], 50, 4096, 0.0)
    cp = t.comm_path_ptr
    for k in range(0, t.n_comm, 2):
        assert np.array_equal(a[cp[k]:cp[k + 1]], b[cp[k]:cp[k + 1]])
    for k in range(1, t.n_comm, 2):
        assert not b[cp[k]:cp[k + 1]].any()


def test_quantized_plan_keeps_the_congestion(oracle_mod):
    """Moving less than one chunk per candidate changes a link's load by at most (number of
    candidates through it) chunks: lambda of the chunked plan stays within that bound."""
    w = W.make_config(1)
    t = w.topo
    iters = 300
    plan = oracle_mod.solve(*t.csr(), w.traffic, w.eps, iters)
    chi = 65536
    flows = oracle_mod.quantize(t.comm_path_ptr, w.traffic, plan["splits"], iters, chi, 0.0)
    load = np.zeros(t.n_links)
    through = np.zeros(t.n_links)
    for p in range(t.n_paths):
        links = t.path_links[t.path_link_ptr[p]:t.path_link_ptr[p + 1]]
        load[links] += flows[p]
        through[links] += 1
    lam_q = (load / t.cap).max()
    assert lam_q <= plan["lam"] + (2 * chi * through / t.cap).max()
