"""GPU parity of nimble_plan_quantize against oracle/quantize_oracle.py, through the C ABI:
the byte flows must be bit-identical."""
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


def gpu_quantize(B, t, demand, splits, iters, chi, theta):
    import torch
    h = B.nimble_topo_create(*t.csr())
    try:
        d = torch.as_tensor(np.ascontiguousarray(demand, dtype=np.float64)).to("cuda:0")
        x = torch.as_tensor(np.ascontiguousarray(splits, dtype=np.float64)).to("cuda:0")
        f = torch.full((t.n_paths,), float("nan"), dtype=torch.float64, device="cuda:0")
        B.nimble_plan_quantize(h, d, x, iters, chi, theta, f)
        torch.cuda.synchronize()
        return f.cpu().numpy()
    finally:
        h.close()


@pytest.mark.parametrize("cfg,iters,chi,theta", [(0, 200, 1 << 20, float(1 << 20)),
                                                 (1, 300, 65536, 0.0),
                                                 (1, 300, 1, float(1 << 22)),
                                                 (3, 100, 1 << 20, float(1 << 20))])
def test_plans_of_the_benchmark_fabrics(oracle_mod, B, cfg, iters, chi, theta):
    w = W.make_config(cfg)
    t = w.topo
    print(f"[quantize] config {cfg} chi={chi}", flush=True)
    h = B.nimble_topo_create(*t.csr())
    try:
        splits, lam = B.plan(h, w.traffic, w.eps, iters)
    finally:
        h.close()
    ref = oracle_mod.quantize(t.comm_path_ptr, w.traffic, splits, iters, chi, theta)
    got = gpu_quantize(B, t, w.traffic, splits, iters, chi, theta)
    assert np.array_equal(got, ref)
    cp = t.comm_path_ptr
    sums = np.add.reduceat(got, cp[:-1])
    assert np.array_equal(sums, w.traffic)


@pytest.mark.parametrize("seed", [1, 2])
def test_random_counts_many_candidates(oracle_mod, B, seed):
    """Ragged candidate lists up to 100 entries with arbitrary counts (not from a solve)."""
    rng = np.random.default_rng(seed)
    t = W.random_topology(rng, 50, 60, 100, 2)
    iters = 977
    splits = np.zeros(t.n_paths)
    cp = t.comm_path_ptr
    for k in range(t.n_comm):
        n = cp[k + 1] - cp[k]
        c = rng.multinomial(iters, rng.dirichlet(np.ones(n) * 0.3))
        splits[cp[k]:cp[k + 1]] = c / iters
    d = rng.integers(0, 1 << 32, size=t.n_comm).astype(np.float64)   # below 2^31 chunks of 3
    d[::7] = 0.0
    for chi, theta in ((4096, 0.0), (1 << 20, float(1 << 24)), (3, 0.0)):
        ref = oracle_mod.quantize(cp, d, splits, iters, chi, theta)
        got = gpu_quantize(B, t, d, splits, iters, chi, theta)
        assert np.array_equal(got, ref)


@pytest.mark.parametrize("max_paths", [2, 3, 7, 12, 16, 25, 33, 64, 65])
@pytest.mark.parametrize("iters", [12, 1 << 25])
def test_every_group_width_with_ties(oracle_mod, B, max_paths, iters):
    """One lane group per pair for up to 64 candidates (group widths 2..64), one thread per pair
    beyond; few distinct counts, so equal remainders are broken by index; the large iteration
    count takes the 64-bit rank keys."""
    rng = np.random.default_rng(100 + max_paths)
    t = W.random_topology(rng, 40, 150, max_paths, 2)
    cp = t.comm_path_ptr
    assert int(np.diff(cp).max()) == max_paths
    splits = np.zeros(t.n_paths)
    unit = iters // 12
    for k in range(t.n_comm):
        n = cp[k + 1] - cp[k]
        c = rng.multinomial(12, np.ones(n) / n) * unit
        c[0] += iters - c.sum()
        splits[cp[k]:cp[k + 1]] = c / iters
    d = rng.integers(0, 1 << 30, size=t.n_comm).astype(np.float64)
    for chi in (1, 4096):
        ref = oracle_mod.quantize(cp, d, splits, iters, chi, 0.0)
        got = gpu_quantize(B, t, d, splits, iters, chi, 0.0)
        assert np.array_equal(got, ref)


def test_too_many_chunks_is_flagged_and_bad_arguments_are_refused(B):
    import torch
    w = W.make_config(0)
    t = w.topo
    d = np.full(t.n_comm, 2.0 ** 40)
    x = np.zeros(t.n_paths)
    x[t.comm_path_ptr[:-1]] = 1.0
    got = gpu_quantize(B, t, d, x, 10, 1, 0.0)              # 2^40 chunks of one byte
    assert np.isnan(got).all()
    h = B.nimble_topo_create(*t.csr())
    dd = torch.zeros(t.n_comm, dtype=torch.float64, device="cuda:0")
    xx = torch.zeros(t.n_paths, dtype=torch.float64, device="cuda:0")
    ff = torch.zeros(t.n_paths, dtype=torch.float64, device="cuda:0")
    try:
        for iters, chi, theta in ((0, 1, 0.0), (10, 0, 0.0), (10, 1, -1.0)):
            with pytest.raises(B.NimbleError) as ei:
                B.nimble_plan_quantize(h, dd, xx, iters, chi, theta, ff)
            assert ei.value.status == B.NIMBLE_ERR_INVALID
    finally:
        h.close()
