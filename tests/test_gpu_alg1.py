"""GPU parity of the batched Algorithm 1 planner against oracle/alg1_oracle.c, through the C ABI:
flows, lambda and sweep counts must be bit-identical."""
import numpy as np
import pytest

from paper_2604_00317_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2604_00317_amd import binding
    binding.load_library(build_if_missing=False)
    return binding


@pytest.fixture(autouse=True, params=["lanes-per-problem", "thread-per-problem"])
def alg1_kernel(request, monkeypatch):
    """Every test runs with the library's own choice of kernel (a lane group per problem where
    the fabric fits it) and with the thread-per-problem kernel forced."""
    if request.param == "thread-per-problem":
        monkeypatch.setenv("NIMBLE_TUNE_ALG1_THREAD_PER_PROBLEM", "1")
    return request.param


def make_topo(B, t, flags=0):
    return B.nimble_topo_create(t.n_links, t.cap, t.n_comm, t.comm_path_ptr, t.n_paths,
                                t.path_link_ptr, t.path_links, flags)


def check(oracle_mod, B, t, demands, phi, chi, max_sweeps=1 << 20):
    demands = np.atleast_2d(np.asarray(demands, dtype=np.float64))
    h = make_topo(B, t)
    try:
        flows, lam, sweeps = B.plan_alg1(h, demands, phi, chi, max_sweeps)
    finally:
        B.nimble_topo_destroy(h)
    for b in range(demands.shape[0]):
        ref = oracle_mod.alg1(*t.csr(), demands[b], phi, chi, max_sweeps)
        assert np.array_equal(flows[b], ref["flows"]), f"problem {b}"
        assert lam[b] == ref["lam"] and sweeps[b] == ref["sweeps"], f"problem {b}"
    return flows, lam, sweeps


def _parallel_links(caps, n_comm=1):
    m = len(caps)
    return W.Topology(n_links=m, cap=np.asarray(caps, dtype=np.float64), n_comm=n_comm,
                      comm_path_ptr=np.arange(n_comm + 1, dtype=np.int32) * m, n_paths=n_comm * m,
                      path_link_ptr=np.arange(n_comm * m + 1, dtype=np.int32),
                      path_links=np.tile(np.arange(m, dtype=np.int32), n_comm),
                      src=np.zeros(n_comm, dtype=np.int32), dst=np.zeros(n_comm, dtype=np.int32),
                      meta=dict(kind="parallel"))


def _gpu_alg1(B, t, demand, phi, chi):
    h = make_topo(B, t)
    try:
        flows, lam, sweeps = B.plan_alg1(h, np.asarray(demand, dtype=np.float64), phi, chi)
    finally:
        B.nimble_topo_destroy(h)
    return flows, lam, sweeps


def test_hand_worked_examples_directly(B):
    """Both kernels against the examples of Algorithm 1 worked by hand -- the same facts that pin
    the CPU oracle (tests/golden/alg1_worked_example.txt, tests/test_alg1_pins.py) -- without
    the oracle in between: the four-sweep example, the Gauss-Seidel schedule, bottleneck versus
    additive cost, chunk multiples with the residual rule, and conservation on a benchmark
    fabric."""
    import os
    golden = os.path.join(os.path.dirname(__file__), "golden", "alg1_worked_example.txt")
    f0, f1, lam0, sw0 = [l for l in open(golden) if l[0] != "#"][0].split()
    flows, lam, sweeps = _gpu_alg1(B, _parallel_links([100.0, 50.0]), [8.0], 0.5, 1.0)
    assert flows.tolist() == [float(f0), float(f1)] and lam == float(lam0) and sweeps == int(sw0)
    # the second pair already sees the first one's load (a Jacobi schedule would not)
    flows, lam, sweeps = _gpu_alg1(B, _parallel_links([10.0, 10.0], 2), [4.0, 4.0], 1.0, 1.0)
    assert flows.tolist() == [4.0, 0.0, 0.0, 4.0] and sweeps == 1 and lam == 0.4
    # bottleneck cost max(0.3, 0.3) = 0.3 beats 0.5; an additive cost (0.6) would not
    t = W.Topology(n_links=3, cap=np.full(3, 10.0), n_comm=3,
                   comm_path_ptr=np.array([0, 1, 2, 4], dtype=np.int32), n_paths=4,
                   path_link_ptr=np.array([0, 2, 3, 4, 6], dtype=np.int32),
                   path_links=np.array([0, 1, 2, 2, 0, 1], dtype=np.int32),
                   src=np.zeros(3, dtype=np.int32), dst=np.zeros(3, dtype=np.int32),
                   meta=dict(kind="tiny"))
    flows, lam, sweeps = _gpu_alg1(B, t, [3.0, 5.0, 1.0], 1.0, 1.0)
    assert flows.tolist() == [3.0, 5.0, 0.0, 1.0] and lam == 0.5
    # d = 10, phi = 0.5, chi = 4: 4, then one chunk of 4 (floor(3/4) = 0), then the residual 2
    flows, lam, sweeps = _gpu_alg1(B, _parallel_links([1.0, 1.0]), [10.0], 0.5, 4.0)
    assert flows.tolist() == [6.0, 4.0] and sweeps == 3
    # conservation and whole chunks on the single node: flows of a pair add up to its demand,
    # every flow but a pair's residual is a multiple of the chunk, lambda is the load maximum
    w = W.make_config(0)
    t, chi = w.topo, float(1 << 20)
    flows, lam, sweeps = _gpu_alg1(B, t, w.traffic, 0.5, chi)
    per_pair = np.add.reduceat(flows, t.comm_path_ptr[:-1])
    assert np.array_equal(per_pair, w.traffic)
    load = np.zeros(t.n_links)
    for p in range(t.n_paths):
        load[t.path_links[t.path_link_ptr[p]:t.path_link_ptr[p + 1]]] += flows[p]
    assert lam == pytest.approx((load / t.cap).max(), rel=1e-14)
    odd = np.add.reduceat((np.mod(flows, chi) != 0).astype(np.int64), t.comm_path_ptr[:-1])
    assert np.all(odd <= 1)


@pytest.mark.parametrize("phi,chi", [(0.5, float(1 << 20)), (0.25, 65536.0), (1.0, 4096.0)])
def test_single_node_batch(oracle_mod, B, phi, chi):
    """The batched single-node workload: 67 problems span two workgroups with a ragged tail."""
    w = W.make_config(2, batch=67)
    print(f"[alg1] batch=67 phi={phi} chi={chi}", flush=True)
    check(oracle_mod, B, w.topo, w.traffic, phi, chi)


def test_zipf_node_and_two_nodes(oracle_mod, B):
    for cfg in (0, 1):
        w = W.make_config(cfg)
        print(f"[alg1] config {cfg}", flush=True)
        check(oracle_mod, B, w.topo, w.traffic, 0.5, float(1 << 20))


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_topologies_and_non_integer_demands(oracle_mod, B, seed):
    rng = np.random.default_rng(seed)
    t = W.random_topology(rng, 40, 30, 9, 4)
    d = rng.random((5, t.n_comm)) * 1e6                  # not integers: still bit-identical
    d[1] = 0.0                                           # a problem without traffic
    d[2, ::2] = 0.0
    print(f"[alg1] random seed={seed}", flush=True)
    flows, lam, sweeps = check(oracle_mod, B, t, d, 0.3, 1000.0)
    assert sweeps[1] == 0 and lam[1] == 0.0


@pytest.mark.parametrize("max_paths", [1, 2, 5, 16, 33, 64, 70])
def test_every_group_width(oracle_mod, B, max_paths):
    """Lane groups of 1 to 64 lanes per problem (several problems per wave, a ragged last
    workgroup); 70 candidates are beyond a wave and take the thread-per-problem kernel."""
    rng = np.random.default_rng(300 + max_paths)
    t = W.random_topology(rng, 25, 12, max_paths, 3)
    nb = 2 * (256 // min(64, max(1, 1 << (max_paths - 1).bit_length()))) + 3
    nb = min(nb, 40)
    d = np.floor(rng.pareto(1.2, (nb, t.n_comm)) * 1e5)
    d[0] = 0.0
    print(f"[alg1] max_paths={max_paths} problems={nb}", flush=True)
    check(oracle_mod, B, t, d, 0.4, 5000.0)


def test_chunk_larger_than_every_demand(oracle_mod, B):
    w = W.make_config(0)
    flows, lam, sweeps = check(oracle_mod, B, w.topo, w.traffic, 0.5, 1e12)
    assert sweeps[0] == 1                                # residual rule: everything at once


def test_sweep_limit_is_reported(oracle_mod, B):
    w = W.make_config(0)
    h = make_topo(B, w.topo)
    try:
        flows, lam, sweeps = B.plan_alg1(h, w.traffic, 0.5, 1.0, max_sweeps=3)
    finally:
        B.nimble_topo_destroy(h)
    assert np.isnan(lam) and sweeps == 3
    with pytest.raises(ValueError):
        oracle_mod.alg1(*w.topo.csr(), w.traffic, 0.5, 1.0, 3)


def test_argument_errors(B):
    import torch
    w = W.make_config(0)
    h = make_topo(B, w.topo)
    d = torch.zeros(w.topo.n_comm, dtype=torch.float64, device="cuda:0")
    f = torch.zeros(w.topo.n_paths, dtype=torch.float64, device="cuda:0")
    lam = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    sw = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    try:
        for phi, chi, ms in ((0.0, 1.0, 10), (1.5, 1.0, 10), (0.5, 0.0, 10), (0.5, 1.0, 0)):
            with pytest.raises(B.NimbleError) as ei:
                B.nimble_alg1_solve_batch(h, 1, d, phi, chi, ms, f, lam, sw)
            assert ei.value.status == B.NIMBLE_ERR_INVALID
    finally:
        B.nimble_topo_destroy(h)
    # a fabric whose per-problem state does not fit in LDS is refused
    big = W.make_config(3)
    h = make_topo(B, big.topo)
    d = torch.zeros(big.topo.n_comm, dtype=torch.float64, device="cuda:0")
    f = torch.zeros(big.topo.n_paths, dtype=torch.float64, device="cuda:0")
    try:
        with pytest.raises(B.NimbleError) as ei:
            B.nimble_alg1_solve_batch(h, 1, d, 0.5, 1.0, 10, f, lam, sw)
        assert ei.value.status == B.NIMBLE_ERR_RANGE
    finally:
        B.nimble_topo_destroy(h)
