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
