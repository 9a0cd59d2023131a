"""GPU parity of nimble_plan_solve_adaptive against oracle/adaptive_oracle.c, through the C ABI."""
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


def gpu_adaptive(B, topo, demand, eps, max_iters, check_every, flags=0, folds=None):
    import torch
    h = B.nimble_topo_create(topo.n_links, topo.cap, topo.n_comm, topo.comm_path_ptr,
                             topo.n_paths, topo.path_link_ptr, topo.path_links, flags)
    try:
        if folds is not None:
            assert h.adaptive_folds == folds
        d = torch.as_tensor(np.ascontiguousarray(demand, dtype=np.float64)).to("cuda:0")
        splits = torch.full((topo.n_paths,), float("nan"), dtype=torch.float64, device="cuda:0")
        lam = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda:0")
        iters, lb = B.nimble_plan_solve_adaptive(h, d, eps, max_iters, check_every, splits, lam)
        return splits.cpu().numpy(), float(lam.item()), iters, lb
    finally:
        h.close()


def check(oracle_mod, B, topo, demand, eps, max_iters, check_every, flags=0, folds=None):
    ref = oracle_mod.solve_adaptive(*topo.csr(), demand, eps, max_iters, check_every, flags=flags)
    splits, lam, iters, lb = gpu_adaptive(B, topo, demand, eps, max_iters, check_every, flags,
                                          folds)
    assert iters == ref["iters"]
    assert lb == ref["lb"]
    assert lam == ref["lam"]
    assert np.array_equal(splits, ref["splits"])
    return ref


@pytest.mark.parametrize("cfg,check_every", [(0, 10), (0, 1), (1, 7), (3, 25)])
def test_stops_where_the_oracle_stops(oracle_mod, B, cfg, check_every):
    w = W.make_config(cfg)
    print(f"[adaptive] config {cfg} check_every={check_every}", flush=True)
    ref = check(oracle_mod, B, w.topo, w.traffic, w.eps, 5000, check_every)
    assert ref["iters"] < 5000 and ref["lam"] <= (1 + w.eps) ** 2 * ref["lb"]


def test_iteration_limit_and_bottleneck_cost(oracle_mod, B):
    w = W.make_config(1)
    check(oracle_mod, B, w.topo, w.traffic, w.eps, 37, 10)             # limit before the gap
    ref = check(oracle_mod, B, w.topo, w.traffic, w.eps, 60, 10, flags=1)
    assert ref["iters"] == 60 and ref["lb"] == 0.0                     # no bound in this mode


def test_tiled_layout_of_the_large_fabric(oracle_mod, B):
    w = W.make_config(4)
    print("[adaptive] config 4, 30 iterations", flush=True)
    check(oracle_mod, B, w.topo, w.traffic, w.eps, 30, 10)


@pytest.mark.parametrize("seed", [3, 4])
def test_random_topologies(oracle_mod, B, seed):
    rng = np.random.default_rng(seed)
    t = W.random_topology(rng, 60, 300, 20, 4)
    d = rng.integers(0, 1 << 24, size=t.n_comm).astype(np.float64)
    check(oracle_mod, B, t, d, 0.1, 400, 5)


@pytest.mark.parametrize("fold", [0, 1])
def test_step_applied_inside_the_next_record_kernel_or_on_its_own(oracle_mod, B, monkeypatch, fold):
    """Where the record kernel can, the step of an iteration is applied inside the record kernel
    of the next one, its prices formed on the fly; a switch read at create forces either way.
    Both must give the oracle's bits: every check period from 1 (a stop test after every
    iteration) up, limits of 1, 2 and 3 iterations, the limit reached on a check and between two
    checks, both cost rules, inline and dictionary records (configuration 4: 30 iterations)."""
    monkeypatch.setenv("NIMBLE_TUNE_ADAPTIVE_FOLD", str(fold))
    w = W.make_config(3)
    for max_iters, check_every in ((1, 1), (2, 1), (3, 2), (40, 1), (40, 7), (50, 25), (60, 100)):
        print(f"[adaptive fold={fold}] config 3 max_iters={max_iters} check_every={check_every}",
              flush=True)
        check(oracle_mod, B, w.topo, w.traffic, w.eps, max_iters, check_every, folds=bool(fold))
    print(f"[adaptive fold={fold}] config 3 to the stop", flush=True)
    ref = check(oracle_mod, B, w.topo, w.traffic, w.eps, 5000, 3, folds=bool(fold))
    assert ref["iters"] < 5000
    print(f"[adaptive fold={fold}] config 3, bottleneck cost", flush=True)
    check(oracle_mod, B, w.topo, w.traffic, w.eps, 30, 10, flags=1, folds=bool(fold))
    w = W.make_config(4)
    print(f"[adaptive fold={fold}] config 4, 30 iterations", flush=True)
    check(oracle_mod, B, w.topo, w.traffic, w.eps, 30, 10, folds=bool(fold))
    rng = np.random.default_rng(11)
    t = W.random_topology(rng, 60, 300, 20, 4)
    d = rng.integers(0, 1 << 24, size=t.n_comm).astype(np.float64)
    print(f"[adaptive fold={fold}] random topology", flush=True)
    check(oracle_mod, B, t, d, 0.1, 200, 4)


def test_default_choice_of_where_the_step_is_applied(B):
    """Folding pays while every record is scanned at once: the 16-node fabric folds, the 64-node
    one (64 records per compute unit) does not."""
    for cfg, folds in ((3, True), (4, False)):
        w = W.make_config(cfg)
        h = B.nimble_topo_create(*w.topo.csr())
        try:
            assert h.adaptive_folds == folds
        finally:
            h.close()


def test_zero_traffic(oracle_mod, B):
    w = W.make_config(0)
    ref = check(oracle_mod, B, w.topo, np.zeros(w.topo.n_comm), 0.1, 40, 5)
    assert ref["iters"] == 0 and ref["lam"] == 0.0


def test_argument_errors(B):
    import torch
    w = W.make_config(0)
    h = B.nimble_topo_create(*w.topo.csr())
    d = torch.zeros(w.topo.n_comm, dtype=torch.float64, device="cuda:0")
    sp = torch.zeros(w.topo.n_paths, dtype=torch.float64, device="cuda:0")
    lam = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    try:
        for eps, mi, ce in ((0.0, 10, 1), (0.1, 0, 1), (0.1, 10, 0)):
            with pytest.raises(B.NimbleError) as ei:
                B.nimble_plan_solve_adaptive(h, d, eps, mi, ce, sp, lam)
            assert ei.value.status == B.NIMBLE_ERR_INVALID
    finally:
        h.close()
