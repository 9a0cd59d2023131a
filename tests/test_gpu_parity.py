"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Bar: splits and lambda within 1e-9 relative (binary64 on both sides).  The arithmetic of both
sides is the same sequence of IEEE operations, so for the integer-valued byte demands of every
benchmark configuration the test also demands the stronger property, exact equality.
"""
import numpy as np
import pytest

from paper_2604_00317_amd import workloads as W

pytestmark = pytest.mark.gpu

RTOL = 1e-9


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a visible MI355X; no fallback path exists")
    from paper_2604_00317_amd import binding
    binding.load_library(build_if_missing=False)
    return binding


def gpu_plan(B, topo, traffic, eps, iters, regime=0, flags=0):
    print(f"[gpu_plan] K={topo.n_comm} P={topo.n_paths} nnz={topo.nnz} E={topo.n_links} "
          f"iters={iters} regime={regime} flags={flags}", flush=True)
    h = B.nimble_topo_create(*topo.csr(), flags=flags)
    try:
        B.nimble_topo_set_regime(h, regime)
        splits, lam = B.plan(h, traffic, eps, iters)
        used = h.regime
    finally:
        h.close()
    return splits, lam, used


def check(oracle_mod, B, topo, traffic, eps, iters, regime=0, flags=0, exact=True):
    ref = oracle_mod.solve(*topo.csr(), traffic, eps, iters, flags=flags)
    splits, lam, used = gpu_plan(B, topo, traffic, eps, iters, regime, flags)
    if regime:
        assert used == regime
    np.testing.assert_allclose(splits, ref["splits"], rtol=RTOL, atol=0)
    assert abs(lam - ref["lam"]) <= RTOL * abs(ref["lam"])
    if exact:
        assert np.array_equal(splits, ref["splits"])
        assert lam == ref["lam"]
    return splits, lam


def _parallel(caps):
    m = len(caps)
    return W.Topology(n_links=m, cap=np.asarray(caps, dtype=np.float64), n_comm=1,
                      comm_path_ptr=np.array([0, m], dtype=np.int32), n_paths=m,
                      path_link_ptr=np.arange(m + 1, dtype=np.int32),
                      path_links=np.arange(m, dtype=np.int32), src=np.zeros(1, dtype=np.int32),
                      dst=np.zeros(1, dtype=np.int32), meta=dict(kind="parallel"))


@pytest.mark.parametrize("regime", [1, 2, 3])
def test_hand_derived_trajectories_directly(B, regime):
    """The HIP path against the facts that pin the oracle, without the oracle in between: the
    hand-derived trajectories on two parallel links (sum cost: the slower link is first taken in
    iteration 15; bottleneck cost: tests/golden/bottleneck_two_links.txt) and the exact round
    robin over equal links."""
    import os
    def counts(t, T, flags=0):
        splits, lam, _ = gpu_plan(B, t, [1e6], 0.1, T, regime, flags)
        return np.rint(splits * T).astype(int).tolist(), lam
    assert counts(_parallel([100e9, 50e9]), 15)[0] == [15, 0]
    assert counts(_parallel([100e9, 50e9]), 16)[0] == [15, 1]
    assert counts(_parallel([100e9, 50e9]), 17)[0] == [16, 1]
    c, lam = counts(_parallel([50e9] * 4), 200)
    assert c == [50] * 4 and lam == pytest.approx(1e6 / (4 * 50e9), rel=1e-14)
    golden = os.path.join(os.path.dirname(__file__), "golden", "bottleneck_two_links.txt")
    rows = {l.split()[0]: [int(float(x)) for x in l.split()[1:]]
            for l in open(golden) if l.split() and l[0] != "#"}
    for key, caps in (("fixed", [100e9, 50e9]), ("fixed_swapped", [50e9, 100e9])):
        want = rows[key]
        for T in (1, 2, 5, len(want)):
            ones = sum(want[:T])
            assert counts(_parallel(caps), T, flags=1)[0] == [T - ones, ones], (key, T)


@pytest.mark.parametrize("regime", [1, 2, 3])
@pytest.mark.parametrize("cfg", [0, 1])
def test_small_configs_full_iterations(oracle_mod, B, cfg, regime):
    w = W.make_config(cfg)
    check(oracle_mod, B, w.topo, w.traffic, w.eps, w.iters, regime)


@pytest.mark.parametrize("regime", [2, 3])
def test_config3_full_iterations(oracle_mod, B, regime):
    w = W.make_config(3)
    check(oracle_mod, B, w.topo, w.traffic, w.eps, w.iters, regime=regime)


@pytest.mark.parametrize("batch", [1, 5, 67])
def test_batched_single_node(oracle_mod, B, batch):
    w = W.make_config(2, batch=batch)
    t = w.topo
    print(f"[batch] batch={batch}", flush=True)
    h = B.nimble_topo_create(*t.csr())
    try:
        assert h.resident_in_registers
        splits, lam = B.plan(h, w.traffic, w.eps, w.iters)
        assert h.regime == B.NIMBLE_REGIME_RESIDENT
    finally:
        h.close()
    for b in range(batch):
        ref = oracle_mod.solve(*t.csr(), w.traffic[b], w.eps, w.iters)
        assert np.array_equal(splits[b], ref["splits"]), b
        assert lam[b] == ref["lam"], b


@pytest.mark.parametrize("regime", [2, 3])
def test_batch_outside_the_resident_regime(oracle_mod, B, regime):
    """Topologies that do not fit LDS (or a forced regime) solve a batch one plan after another
    on the stream, reusing the topology's workspace: every plan must still match the oracle."""
    w = W.make_config(2, batch=3)
    t = w.topo
    h = B.nimble_topo_create(*t.csr())
    try:
        B.nimble_topo_set_regime(h, regime)
        splits, lam = B.plan(h, w.traffic, w.eps, 60)
        assert h.regime == regime
    finally:
        h.close()
    for b in range(3):
        ref = oracle_mod.solve(*t.csr(), w.traffic[b], w.eps, 60)
        assert np.array_equal(splits[b], ref["splits"]), b
        assert lam[b] == ref["lam"], b


def _batch_traffic(w, n):
    """n demand vectors for the fabric of w: its own and scaled, thinned and zero variants."""
    rng = np.random.default_rng(7)
    rows = [w.traffic]
    for b in range(1, n):
        d = np.floor(w.traffic / (b + 1))
        d[rng.random(d.size) < 0.1 * b] = 0.0
        rows.append(d)
    if n > 2:
        rows[-1] = np.zeros_like(w.traffic)
    return np.stack(rows)


@pytest.mark.parametrize("env", [{}, {"NIMBLE_TUNE_NO_CHOICE_LOG": "1"},
                                 {"NIMBLE_TUNE_NO_LINK_BLOCKS": "1"},
                                 {"NIMBLE_TUNE_TILES": "1", "NIMBLE_TUNE_TILE_MIN_ITEMS": "24"},
                                 {"NIMBLE_TUNE_RECORD_DICT": "1"},
                                 {"NIMBLE_TUNE_RECORD_LANE_MAJOR": "0"},
                                 {"NIMBLE_TUNE_NO_RECORDS": "1"},
                                 {"NIMBLE_TUNE_BATCH_KERNEL": "1"}],
                         ids=["default", "counters", "separate-update", "tiles", "dictionary",
                              "record-major", "untiled", "plan-by-plan-kernel"])
# (one more variant below: the single-plan reduce + update kernel for every plan of a batch)
def test_streamed_batch_shares_every_launch(oracle_mod, B, monkeypatch, env):
    """A batch of plans on a fabric that is streamed: with room reserved for them the plans of a
    batch run side by side in every kernel launch (one state block and one range of log rows
    each).  Every plan must match the oracle, in every layout the streaming kernels know, with
    the whole batch in one group, in groups of two (the last one short), and bottleneck cost."""
    for name, value in env.items():
        monkeypatch.setenv(name, value)
    import torch
    for cfg, iters, n, flags in ((3, 40, 5, 0), (1, 60, 4, 1)):
        w = W.make_config(cfg)
        t = w.topo
        tr = _batch_traffic(w, n)
        refs = [oracle_mod.solve(*t.csr(), tr[b], w.eps, iters, flags=flags) for b in range(n)]
        for group in (n, 2):
            print(f"[batch] cfg={cfg} n={n} group={group} env={env}", flush=True)
            # (the 16-node fabric, whole batch in one group: on a topology laid out for batches)
            h = B.nimble_topo_create(*t.csr(),
                                     flags=flags | (B.NIMBLE_LAYOUT_BATCH if group == n and cfg == 3
                                                    else 0))
            try:
                B.nimble_topo_set_regime(h, B.NIMBLE_REGIME_STREAM)
                B.nimble_topo_reserve_batch(h, group, iters)
                d = torch.as_tensor(tr.reshape(-1)).to("cuda:0")
                splits = torch.full((n * t.n_paths,), float("nan"), dtype=torch.float64,
                                    device="cuda:0")
                lam = torch.full((n,), float("nan"), dtype=torch.float64, device="cuda:0")
                B.nimble_plan_solve_batch(h, n, d, w.eps, iters, splits, lam)
                torch.cuda.synchronize()
                sp = splits.cpu().numpy().reshape(n, t.n_paths)
                la = lam.cpu().numpy()
                # a single plan afterwards still uses block 0 alone
                one_s = torch.full((t.n_paths,), float("nan"), dtype=torch.float64, device="cuda:0")
                one_l = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda:0")
                B.nimble_plan_solve(h, d[t.n_comm:2 * t.n_comm].contiguous(), w.eps, iters, one_s,
                                    one_l)
                torch.cuda.synchronize()
            finally:
                h.close()
            for b in range(n):
                assert np.array_equal(sp[b], refs[b]["splits"]), (cfg, group, b)
                assert la[b] == refs[b]["lam"], (cfg, group, b)
            assert np.array_equal(one_s.cpu().numpy(), refs[1]["splits"])
            assert float(one_l.item()) == refs[1]["lam"]


@pytest.mark.parametrize("flags", [0, 1])
@pytest.mark.parametrize("seed,E,K,pm,lm,in_regs", [(21, 30, 25, 8, 2, True),
                                                    (22, 64, 64, 5, 2, True),
                                                    (23, 100, 70, 8, 1, True),
                                                    (24, 12, 9, 3, 2, True),
                                                    (25, 130, 100, 8, 2, True),
                                                    (26, 30, 25, 9, 2, False),
                                                    (27, 30, 25, 8, 3, False),
                                                    (28, 6, 60, 8, 2, False)])
def test_resident_regime_register_and_lds_kernels(oracle_mod, B, monkeypatch, seed, E, K, pm, lm,
                                                  in_regs, flags):
    """Small fabrics (at most 8 candidates of 2 links, 16 pairs per link) keep the topology in
    registers; one candidate, one link or one pair more and the LDS kernel runs.  Forcing the
    LDS kernel on the small ones gives the same bits."""
    rng = np.random.default_rng(seed)
    t = W.random_topology(rng, E, K, pm, lm)
    d = np.floor(rng.pareto(1.1, K) * 1e6)
    d[rng.integers(0, K)] = 0.0
    h = B.nimble_topo_create(*t.csr(), flags=flags)
    try:
        assert h.resident_in_registers == in_regs
    finally:
        h.close()
    check(oracle_mod, B, t, d, 0.07, 60, 1, flags)
    if in_regs:
        monkeypatch.setenv("NIMBLE_TUNE_RESIDENT_GENERIC", "1")
        h = B.nimble_topo_create(*t.csr(), flags=flags)
        try:
            assert not h.resident_in_registers
        finally:
            h.close()
        check(oracle_mod, B, t, d, 0.07, 60, 1, flags)


def test_resident_regime_with_more_commodities_and_links_than_threads(oracle_mod, B):
    """A 35-GPU mesh with two candidates per pair: K = E = 1190, lists short enough for the
    register kernel but more commodities and links than a workgroup has threads.  The resident
    regime must stride (LDS kernel): every commodity routed, every link priced."""
    t = W.two_candidate_mesh(35)
    rng = np.random.default_rng(34)
    d = np.floor(rng.pareto(1.1, t.n_comm) * 1e6)
    h = B.nimble_topo_create(*t.csr())
    try:
        assert not h.resident_in_registers
    finally:
        h.close()
    for flags in (0, 1):
        check(oracle_mod, B, t, d, 0.07, 40, 1, flags)
        check(oracle_mod, B, t, d, 0.07, 40, 0, flags)     # whatever the library picks itself


def test_regime_chosen_from_batch_size_and_row_lengths(oracle_mod, B, monkeypatch):
    """The two-node fabric fits the resident regime: one plan, or a few, get a workgroup each
    whose lanes share commodities and links; same bits as the oracle, one plan or four.  With
    only the thread-per-commodity kernel to choose from (its rail links carry 64 pairs each: one
    thread walking such a row is slower than two short kernels per iteration) one plan is
    streamed and a batch runs side by side in the resident regime."""
    w = W.make_config(1)
    t = w.topo
    iters = 50
    tr = np.stack([w.traffic, np.floor(w.traffic / 2), np.floor(w.traffic / 5),
                   np.zeros_like(w.traffic)])
    refs = [oracle_mod.solve(*t.csr(), tr[b], w.eps, iters) for b in range(4)]
    for generic, single in ((False, B.NIMBLE_REGIME_RESIDENT), (True, B.NIMBLE_REGIME_STREAM)):
        if generic:
            monkeypatch.setenv("NIMBLE_TUNE_RESIDENT_GENERIC", "1")
        h = B.nimble_topo_create(*t.csr())
        try:
            splits, lam = B.plan(h, tr[0], w.eps, iters)
            assert h.regime == single
            assert np.array_equal(splits, refs[0]["splits"]) and lam == refs[0]["lam"]
            splits, lam = B.plan(h, tr, w.eps, iters)
            assert h.regime == B.NIMBLE_REGIME_RESIDENT
            for b in range(4):
                assert np.array_equal(splits[b], refs[b]["splits"]), b
                assert lam[b] == refs[b]["lam"], b
        finally:
            h.close()


@pytest.mark.parametrize("flags", [0, 1])
@pytest.mark.parametrize("seed,E,K,pm,lm,kind", [(41, 200, 60, 2, 5, 4), (42, 200, 60, 5, 5, 4),
                                                 (43, 250, 60, 12, 4, 4), (44, 256, 100, 30, 3, 4),
                                                 (45, 256, 60, 60, 2, 4), (46, 257, 60, 12, 4, 3),
                                                 (47, 200, 60, 12, 6, 3), (48, 40, 600, 12, 3, 3)])
def test_cooperative_resident_kernels(oracle_mod, B, seed, E, K, pm, lm, kind, flags):
    """One plan, and a batch of three, on the kernels whose lanes share commodities and links:
    with the lists in registers (kind 4: paths of at most 5 links, at most 256 links, rows of
    at most 64 pairs, few enough commodities) for 2 to 64 lanes per commodity, and with the
    lists in LDS (kind 3) one link, one step or one long row beyond that."""
    rng = np.random.default_rng(seed)
    t = W.random_topology(rng, E, K, pm, lm)
    assert B.nimble_host_resident_kernel(t.n_links, t.n_comm, t.comm_path_ptr, t.n_paths,
                                         t.path_link_ptr, t.path_links) == kind
    d = np.floor(rng.pareto(1.1, (3, K)) * 1e6)
    d[1, ::5] = 0.0
    check(oracle_mod, B, t, d[0], 0.07, 50, 1, flags)
    h = B.nimble_topo_create(*t.csr(), flags=flags)
    try:
        B.nimble_topo_set_regime(h, 1)
        splits, lam = B.plan(h, d, 0.07, 30)
    finally:
        h.close()
    for b in range(3):
        ref = oracle_mod.solve(*t.csr(), d[b], 0.07, 30, flags=flags)
        assert np.array_equal(splits[b], ref["splits"]) and lam[b] == ref["lam"], b


def test_resident_kernels_on_either_side_of_the_cooperative_limit(oracle_mod, B):
    """Up to 256 plans of the two-node fabric get a workgroup each (lanes share commodities and
    links); one plan more and all of them run on the thread-per-commodity kernel, several to a
    workgroup.  Both must give the oracle's plans."""
    w = W.make_config(1)
    t = w.topo
    iters = 30
    for n in (256, 257):
        tr = np.stack([np.floor(w.traffic / (1 + b % 7)) for b in range(n)])
        h = B.nimble_topo_create(*t.csr())
        try:
            splits, lam = B.plan(h, tr, w.eps, iters)
            assert h.regime == B.NIMBLE_REGIME_RESIDENT
        finally:
            h.close()
        for b in (0, 1, 6, n - 1):
            ref = oracle_mod.solve(*t.csr(), tr[b], w.eps, iters)
            assert np.array_equal(splits[b], ref["splits"]), (n, b)
            assert lam[b] == ref["lam"], (n, b)


def test_batched_single_node_with_the_lds_kernel(oracle_mod, B, monkeypatch):
    monkeypatch.setenv("NIMBLE_TUNE_RESIDENT_GENERIC", "1")
    w = W.make_config(2, batch=5)
    t = w.topo
    h = B.nimble_topo_create(*t.csr())
    try:
        assert not h.resident_in_registers
        splits, lam = B.plan(h, w.traffic, w.eps, w.iters)
        assert h.regime == B.NIMBLE_REGIME_RESIDENT
    finally:
        h.close()
    for b in range(5):
        ref = oracle_mod.solve(*t.csr(), w.traffic[b], w.eps, w.iters)
        assert np.array_equal(splits[b], ref["splits"]), b
        assert lam[b] == ref["lam"], b


@pytest.mark.parametrize("regime", [1, 2, 3])
@pytest.mark.parametrize("flags", [0, 1])
@pytest.mark.parametrize("seed,E,K,pm,lm", [(1, 7, 3, 4, 3), (2, 40, 130, 9, 5),
                                            (3, 300, 1000, 20, 6), (4, 64, 65, 33, 4),
                                            (5, 90, 17, 100, 7), (6, 1, 5, 1, 1),
                                            (7, 500, 3000, 12, 2), (8, 50, 40, 127, 2),
                                            (9, 30, 200, 64, 1)])
def test_random_ragged_topologies(oracle_mod, B, seed, E, K, pm, lm, flags, regime):
    rng = np.random.default_rng(seed)
    t = W.random_topology(rng, E, K, pm, lm)
    d = np.floor(rng.pareto(1.1, K) * 1e6)
    d[rng.integers(0, K)] = 0.0
    if regime == 1 and K >= 1000:
        pytest.skip("per-plan state exceeds the LDS budget of the resident regime")
    check(oracle_mod, B, t, d, 0.07, 60, regime, flags)


@pytest.mark.parametrize("regime", [1, 2, 3])
def test_paths_too_long_for_records_use_the_untiled_kernel(oracle_mod, B, regime):
    """Paths of 70 links do not fit the 4 KiB forward records, so the streaming regime falls
    back to the untiled path-cost kernel; paths longer than the unrolled prefix take its tail
    loop."""
    rng = np.random.default_rng(33)
    E, K, npth, ln = 80, 3, 100, 70
    cap = rng.choice([50.0, 100.0], size=E) * 1e9
    pl = np.concatenate([rng.choice(E, size=ln, replace=False) for _ in range(K * npth)])
    t = W.Topology(n_links=E, cap=cap, n_comm=K,
                   comm_path_ptr=(np.arange(K + 1) * npth).astype(np.int32), n_paths=K * npth,
                   path_link_ptr=(np.arange(K * npth + 1) * ln).astype(np.int32),
                   path_links=pl.astype(np.int32), src=np.zeros(K, np.int32),
                   dst=np.zeros(K, np.int32))
    d = np.array([3e6, 7e6, 1e6])
    check(oracle_mod, B, t, d, 0.1, 80, regime)


@pytest.mark.parametrize("regime", [1, 2, 3])
def test_edge_cases(oracle_mod, B, regime):
    t = W.build_fabric(1, 4)
    check(oracle_mod, B, t, np.zeros(t.n_comm), 0.1, 10, regime)          # all-zero traffic
    d = np.zeros(t.n_comm)
    d[5] = 123456789.0
    check(oracle_mod, B, t, d, 0.5, 1, regime)                             # one iteration
    check(oracle_mod, B, t, d, 0.5, 1000, regime)                          # largest step
    big = np.full(t.n_comm, float(2 ** 40))
    check(oracle_mod, B, t, big, 0.1, 40, regime)
    # bottleneck cost on the structured fabric
    w = W.make_config(1)
    check(oracle_mod, B, w.topo, w.traffic, w.eps, 120, regime, flags=1)


@pytest.mark.parametrize("flags", [0, 1])
@pytest.mark.parametrize("env", [{"NIMBLE_TUNE_RECORD_TABLE16": "0"},
                                 {"NIMBLE_TUNE_RECORD_LANE_MAJOR": "0"},
                                 {"NIMBLE_TUNE_RECORD_LANE_MAJOR": "0",
                                  "NIMBLE_TUNE_NO_CHOICE_LOG": "1"},
                                 {"NIMBLE_TUNE_NO_CHOICE_LOG": "1"},
                                 {"NIMBLE_TUNE_RECORD_AROUND_L2": "1"},
                                 {"NIMBLE_TUNE_RECORD_AROUND_L2": "1",
                                  "NIMBLE_TUNE_RECORD_TABLE16": "0"},
                                 {"NIMBLE_TUNE_RECORD_DICT": "0"},
                                 {"NIMBLE_TUNE_RECORD_DICT": "0",
                                  "NIMBLE_TUNE_RECORD_AROUND_L2": "1"},
                                 {"NIMBLE_TUNE_RECORD_DICT": "1"},
                                 {"NIMBLE_TUNE_RECORD_DICT": "1",
                                  "NIMBLE_TUNE_RECORD_AROUND_L2": "1"},
                                 {"NIMBLE_TUNE_RECORD_DICT": "1",
                                  "NIMBLE_TUNE_NO_CHOICE_LOG": "1"},
                                 {"NIMBLE_TUNE_RECORD_DICT": "1",
                                  "NIMBLE_TUNE_RECORDS_PER_WAVE": "3"},
                                 {"NIMBLE_TUNE_RECORD_PRODUCT_QUADS": "0"},
                                 {"NIMBLE_TUNE_RECORD_PRODUCT_QUADS": "0",
                                  "NIMBLE_TUNE_RECORD_DICT": "1"}],
                         ids=["lane-major-32", "record-major", "record-major-counters",
                              "lane-major-16-counters", "lane-major-16-around-l2",
                              "lane-major-32-around-l2", "lane-major-16-inline",
                              "lane-major-16-inline-around-l2", "dictionary",
                              "dictionary-around-l2", "dictionary-counters",
                              "dictionary-runs-of-3", "inline-twenty-reads-per-quad",
                              "dictionary-twenty-reads-per-quad"])
def test_every_forward_record_format(oracle_mod, B, monkeypatch, env, flags):
    """The default on these fabrics is lane-major record bodies with 16-bit link tables, kept
    once each in a dictionary where records share them (the 16-node fabric) and inline otherwise;
    both are forced here on every fabric, the ragged one included, where no two records share a
    body.  The 32-bit table (fabrics of more than 65535 links) and the record-major body (more than five
    links per path, or fewer than nine candidates per commodity) must give the same plans, with
    the choice log and with per-path counters.  Records that exceed the L2 are fetched with
    loads that bypass it; the switch forces those loads on fabrics of any size.  Quads of four
    candidates that differ only in (egress, ingress) are stored in a shape of which the kernel
    reads 9 prices instead of 20 (the default on these fabrics); the last two cases switch that
    off."""
    for name, value in env.items():
        monkeypatch.setenv(name, value)
    for cfg, iters in ((1, 120), (3, 60)):
        w = W.make_config(cfg)
        check(oracle_mod, B, w.topo, w.traffic, w.eps, iters, regime=2, flags=flags)
    # ragged: 1 to 40 candidates of one or two links, commodities without traffic
    rng = np.random.default_rng(77)
    t = W.random_topology(rng, 120, 900, 40, 2)
    d = np.floor(rng.pareto(1.1, t.n_comm) * 1e6)
    d[::9] = 0.0
    check(oracle_mod, B, t, d, 0.07, 50, 2, flags)


def test_streaming_regime_without_choice_log(oracle_mod, B, monkeypatch):
    """When the per-iteration choice log is unavailable the streaming regime counts per path
    every iteration instead; both ways must give the same plan."""
    monkeypatch.setenv("NIMBLE_TUNE_NO_CHOICE_LOG", "1")
    for cfg, iters in ((1, 300), (3, 120)):
        w = W.make_config(cfg)
        check(oracle_mod, B, w.topo, w.traffic, w.eps, iters, regime=2)


def test_streaming_regime_with_separate_reduce_and_update(oracle_mod, B, monkeypatch):
    """Topologies cut into link blocks run the link-load reduce and the length update as one
    kernel; with the blocks switched off the same topologies take the two separate kernels
    (the path every topology with single pairs uses).  Both must give the oracle's plan."""
    monkeypatch.setenv("NIMBLE_TUNE_NO_LINK_BLOCKS", "1")
    for cfg, iters in ((0, 200), (1, 300), (3, 120)):
        w = W.make_config(cfg)
        check(oracle_mod, B, w.topo, w.traffic, w.eps, iters, regime=2)


@pytest.mark.parametrize("passes", [1, 2, 64])
def test_link_block_sizes(oracle_mod, B, monkeypatch, passes):
    """Link blocks of one pass (a block per large row), two passes and one huge block size."""
    monkeypatch.setenv("NIMBLE_TUNE_BLOCK_PASSES", str(passes))
    for cfg, iters in ((1, 300), (3, 60)):
        w = W.make_config(cfg)
        check(oracle_mod, B, w.topo, w.traffic, w.eps, iters, regime=2)
        check(oracle_mod, B, w.topo, w.traffic, w.eps, iters, regime=2, flags=1)


@pytest.mark.parametrize("min_items", [1, 24, 128])
def test_tiled_reverse_layout(oracle_mod, B, monkeypatch, min_items):
    """Dense (link, window) pieces instead of octets, forced on for small fabrics and ragged
    random instances at several piece thresholds, in both regimes that stream the layout."""
    monkeypatch.setenv("NIMBLE_TUNE_TILES", "1")
    monkeypatch.setenv("NIMBLE_TUNE_TILE_MIN_ITEMS", str(min_items))
    for cfg, iters in ((0, 200), (1, 300), (3, 60)):
        w = W.make_config(cfg)
        for regime in (2, 3):
            check(oracle_mod, B, w.topo, w.traffic, w.eps, iters, regime=regime)
        check(oracle_mod, B, w.topo, w.traffic, w.eps, iters, regime=2, flags=1)
    for seed, E, K, pm, lm in ((5, 90, 17, 100, 7), (11, 60, 1500, 6, 3), (12, 300, 700, 31, 2)):
        rng = np.random.default_rng(seed)
        t = W.random_topology(rng, E, K, pm, lm)
        d = rng.integers(0, 1 << 30, size=t.n_comm).astype(np.float64)
        check(oracle_mod, B, t, d, 0.1, 40, regime=2)


@pytest.mark.parametrize("env", [{"NIMBLE_TUNE_LINK_GROUPS": "0"}, {"NIMBLE_TUNE_GROUP_BLOCKS": "1"},
                                 {"NIMBLE_TUNE_GROUP_BLOCKS": "7", "NIMBLE_TUNE_GROUP_WAVES": "4"},
                                 {"NIMBLE_TUNE_GROUP_BLOCKS": "40", "NIMBLE_TUNE_GROUP_WAVES": "16"},
                                 {"NIMBLE_TUNE_GROUP_BLOCKS": "5000", "NIMBLE_TUNE_GROUP_WAVES": "8"}],
                         ids=["no-groups", "one-block", "seven-blocks-4-waves",
                              "forty-blocks-16-waves", "a-block-per-group-8-waves"])
def test_link_groups_reduce_and_update_in_one_launch(oracle_mod, B, monkeypatch, env):
    """A tiled layout whose links are cut into groups runs the link-load reduce and the length
    update of a block of groups in one workgroup (partial sums in LDS).  Any number of blocks
    and any workgroup size must give the oracle's plan, and so must the same layout without
    groups (two kernels)."""
    monkeypatch.setenv("NIMBLE_TUNE_TILES", "1")
    monkeypatch.setenv("NIMBLE_TUNE_TILE_MIN_ITEMS", "24")
    for name, value in env.items():
        monkeypatch.setenv(name, value)
    for cfg, iters in ((1, 300), (3, 60)):
        w = W.make_config(cfg)
        print(f"[groups] cfg={cfg} env={env}", flush=True)
        check(oracle_mod, B, w.topo, w.traffic, w.eps, iters, regime=2)
        check(oracle_mod, B, w.topo, w.traffic, w.eps, iters, regime=2, flags=1)
    rng = np.random.default_rng(12)
    t = W.random_topology(rng, 300, 700, 31, 2)
    d = rng.integers(0, 1 << 30, size=t.n_comm).astype(np.float64)
    check(oracle_mod, B, t, d, 0.1, 40, regime=2)


def test_row_too_long_for_a_link_block(oracle_mod, B):
    """600 000 single-path commodities on one link: the row needs more partial-sum slots than a
    link block holds, so the streaming regime runs the separate reduce and update kernels."""
    K, E = 600_000, 3
    cp = np.arange(K + 1, dtype=np.int32)
    pl = np.zeros(K, dtype=np.int32)
    pl[::1000] = 2
    topo = W.Topology(n_links=E, cap=np.array([100e9, 50e9, 25e9]), n_comm=K, comm_path_ptr=cp,
                      n_paths=K, path_link_ptr=cp.copy(), path_links=pl,
                      src=np.zeros(K, dtype=np.int32), dst=np.zeros(K, dtype=np.int32),
                      meta=dict(kind="one hot link"))
    d = np.random.default_rng(3).integers(1, 1 << 20, size=K).astype(np.float64)
    check(oracle_mod, B, topo, d, 0.1, 5, regime=2)


def test_non_integer_demands(oracle_mod, B, monkeypatch):
    """The resident kernel that gives a thread a whole link adds loads in the sequential order,
    so it is exact for any demands; the cooperative resident kernel (a few plans: 16 lanes per
    link) and the streaming regimes sum in a fixed tree: run-to-run identical, equal to the
    oracle up to the rounding of the load sums."""
    w = W.make_config(1)
    d = w.traffic * (1.0 + np.random.default_rng(0).random(w.topo.n_comm))
    monkeypatch.setenv("NIMBLE_TUNE_RESIDENT_GENERIC", "1")
    check(oracle_mod, B, w.topo, d, w.eps, 100, regime=1, exact=True)
    monkeypatch.delenv("NIMBLE_TUNE_RESIDENT_GENERIC")
    ref = oracle_mod.solve(*w.topo.csr(), d, w.eps, 100)
    t = w.topo
    for regime in (1, 2, 3):
        a = gpu_plan(B, t, d, w.eps, 100, regime=regime)
        b = gpu_plan(B, t, d, w.eps, 100, regime=regime)
        assert np.array_equal(a[0], b[0]) and a[1] == b[1]
        assert abs(a[1] - ref["lam"]) <= 1e-6 * ref["lam"]
        # whatever the rounding of the load sums did to a choice here or there, the plan is a
        # plan: whole iterations per candidate, fractions of a commodity adding up to one, and
        # lambda the congestion of these very fractions
        counts = np.round(a[0] * 100)
        assert np.array_equal(a[0], counts / 100.0)
        per_comm = np.add.reduceat(a[0], t.comm_path_ptr[:-1])
        np.testing.assert_allclose(per_comm, 1.0, rtol=0, atol=1e-12)
        load = np.zeros(t.n_links)
        flow = a[0] * np.repeat(d, np.diff(t.comm_path_ptr))
        np.add.at(load, t.path_links, np.repeat(flow, np.diff(t.path_link_ptr)))
        assert abs((load / t.cap).max() - a[1]) <= 1e-9 * a[1]
        # (few commodities may have chosen differently from the oracle in some iteration)
        assert np.mean(a[0] != ref["splits"]) < 0.05


@pytest.mark.parametrize("scale", [2.0 ** -10, 2.0 ** -40, 3.0 * 2.0 ** 20])
def test_demands_on_a_power_of_two_grid_are_exact_in_every_regime(oracle_mod, B, scale):
    """Load sums are exact, in any order, whenever all demands are whole multiples of one power
    of two and their total stays below 2^53 of those units: fractional byte counts on a binary
    grid (and counts in other units) are therefore bit-identical to the oracle in the regimes
    that add in a tree as well."""
    for cfg, iters in ((1, 120), (3, 40)):
        w = W.make_config(cfg)
        d = np.floor(w.traffic / 7.0) * scale
        for regime in ((1, 2, 3) if cfg == 1 else (2,)):
            check(oracle_mod, B, w.topo, d, w.eps, iters, regime=regime, exact=True)


def test_argument_errors_on_device(B):
    import torch
    t = W.build_fabric(1, 4)
    h = B.nimble_topo_create(*t.csr())
    try:
        d = torch.zeros(t.n_comm, dtype=torch.float64, device="cuda:0")
        s = torch.zeros(t.n_paths, dtype=torch.float64, device="cuda:0")
        lam = torch.zeros(1, dtype=torch.float64, device="cuda:0")
        for eps, iters, status in [(0.0, 10, B.NIMBLE_ERR_INVALID), (0.6, 10, B.NIMBLE_ERR_INVALID),
                                   (float("nan"), 10, B.NIMBLE_ERR_INVALID),
                                   (0.1, 0, B.NIMBLE_ERR_INVALID), (0.5, 2000, B.NIMBLE_ERR_RANGE)]:
            with pytest.raises(B.NimbleError) as ei:
                B.nimble_plan_solve(h, d, eps, iters, s, lam)
            assert ei.value.status == status
        import ctypes
        st = B.load_library().nimble_plan_solve_batch(
            h.handle, 0, ctypes.c_void_p(d.data_ptr()), 0.1, 10, ctypes.c_void_p(s.data_ptr()),
            ctypes.c_void_p(lam.data_ptr()), None)
        assert st == B.NIMBLE_ERR_INVALID
        B.nimble_plan_solve(h, d, 0.1, 10, s, lam)       # still usable after errors
        torch.cuda.synchronize()
        assert float(lam.item()) == 0.0
    finally:
        h.close()


@pytest.mark.parametrize("cfg,iters", [(1, 40), (3, 60)])
def test_a_solve_can_be_captured_in_a_graph(oracle_mod, B, cfg, iters):
    """After one eager solve (which sizes the workspace) a solve only enqueues kernels, so a
    caller may capture it; every replay, with eager solves of other traffic in between, gives
    the oracle's bits again."""
    import torch
    w = W.make_config(cfg)
    t = w.topo
    ref = oracle_mod.solve(*t.csr(), w.traffic, w.eps, iters)
    other = np.floor(w.traffic / 3.0)
    ref_other = oracle_mod.solve(*t.csr(), other, w.eps, iters)
    h = B.nimble_topo_create(*t.csr())
    try:
        d_tr = torch.as_tensor(w.traffic).to("cuda:0")
        d_ot = torch.as_tensor(other).to("cuda:0")
        d_sp = torch.empty(t.n_paths, dtype=torch.float64, device="cuda:0")
        d_la = torch.empty(1, dtype=torch.float64, device="cuda:0")
        d_sp2 = torch.empty_like(d_sp)
        d_la2 = torch.empty_like(d_la)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            B.nimble_plan_solve(h, d_tr, w.eps, iters, d_sp, d_la)
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                B.nimble_plan_solve(h, d_tr, w.eps, iters, d_sp, d_la)
        torch.cuda.synchronize()
        for replay in range(3):
            d_sp.zero_()
            d_la.zero_()
            B.nimble_plan_solve(h, d_ot, w.eps, iters, d_sp2, d_la2)      # eager, in between
            torch.cuda.synchronize()
            assert np.array_equal(d_sp2.cpu().numpy(), ref_other["splits"]), replay
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(d_sp.cpu().numpy(), ref["splits"]), replay
            assert float(d_la.item()) == ref["lam"], replay
    finally:
        h.close()


def test_streaming_read_helper(B):
    """The bandwidth probe of the benchmark: runs, leaves its buffer alone, refuses bad input."""
    import torch
    buf = torch.arange(1 << 16, dtype=torch.float64, device="cuda:0")
    sink = torch.zeros(2, dtype=torch.float64, device="cuda:0")
    B.nimble_debug_stream_read(buf, buf.numel() * 8, 3, sink)
    B.nimble_debug_stream_read(buf, 16, 1, sink)
    torch.cuda.synchronize()
    assert torch.equal(buf, torch.arange(1 << 16, dtype=torch.float64, device="cuda:0"))
    with pytest.raises(ValueError):
        B.nimble_debug_stream_read(buf, buf.numel() * 8 + 16, 1, sink)
    with pytest.raises(B.NimbleError):
        B.nimble_debug_stream_read(buf, 8, 1, sink)
    with pytest.raises(B.NimbleError):
        B.nimble_debug_stream_read(buf[1:], 64, 1, sink)      # 8-byte aligned only


def test_solve_on_side_stream_and_reuse(oracle_mod, B):
    import torch
    w = W.make_config(1)
    t = w.topo
    h = B.nimble_topo_create(*t.csr())
    try:
        B.nimble_topo_set_regime(h, B.NIMBLE_REGIME_STREAM)
        stream = torch.cuda.Stream()
        d = torch.as_tensor(w.traffic).to("cuda:0")
        s = torch.empty(t.n_paths, dtype=torch.float64, device="cuda:0")
        lam = torch.empty(1, dtype=torch.float64, device="cuda:0")
        torch.cuda.synchronize()
        for iters in (50, 20):                      # second solve re-initialises the workspace
            B.nimble_plan_solve(h, d, w.eps, iters, s, lam, stream=stream)
            stream.synchronize()
            ref = oracle_mod.solve(*t.csr(), w.traffic, w.eps, iters)
            assert np.array_equal(s.cpu().numpy(), ref["splits"])
            assert float(lam.item()) == ref["lam"]
    finally:
        h.close()


def test_device_allocation_failures_leave_nothing_behind(oracle_mod, B):
    """Every device allocation of nimble_topo_create is made to fail in turn (test hook): the
    call must return NIMBLE_ERR_ALLOC with nothing left allocated, and the first create that is
    spared must work.  The same for the calls that grow the workspace later."""
    import ctypes
    import torch
    lib = B.load_library()
    w = W.make_config(1)
    t = w.topo
    base = lib.nimble_debug_live_allocations()
    made = None
    for n in range(400):
        assert lib.nimble_debug_fail_allocation(n) == B.NIMBLE_OK
        try:
            made = B.nimble_topo_create(*t.csr())
            break
        except B.NimbleError as err:
            assert err.status == B.NIMBLE_ERR_ALLOC, (n, str(err))
            assert lib.nimble_debug_live_allocations() == base, n
    lib.nimble_debug_fail_allocation(-1)
    assert made is not None and n >= 20          # a create makes dozens of allocations
    try:
        ref = oracle_mod.solve(*t.csr(), w.traffic, w.eps, 50)
        splits, lam = B.plan(made, w.traffic, w.eps, 50)
        assert np.array_equal(splits, ref["splits"]) and lam == ref["lam"]
        held = lib.nimble_debug_live_allocations()
        # growing the log, the batch state and the adaptive workspace under failure
        for call in (lambda: B.nimble_topo_reserve(made, 5000),
                     lambda: B.nimble_topo_reserve_batch(made, 3, 100)):
            lib.nimble_debug_fail_allocation(0)
            with pytest.raises(B.NimbleError) as ei:
                call()
            assert ei.value.status == B.NIMBLE_ERR_ALLOC
            assert lib.nimble_debug_live_allocations() <= held
            lib.nimble_debug_fail_allocation(-1)
        d = torch.as_tensor(w.traffic).to("cuda:0")
        sp = torch.zeros(t.n_paths, dtype=torch.float64, device="cuda:0")
        la = torch.zeros(1, dtype=torch.float64, device="cuda:0")
        for n in range(3):
            before = lib.nimble_debug_live_allocations()
            lib.nimble_debug_fail_allocation(n)
            with pytest.raises(B.NimbleError) as ei:
                B.nimble_plan_solve_adaptive(made, d, w.eps, 200, 10, sp, la)
            assert ei.value.status == B.NIMBLE_ERR_ALLOC
            assert lib.nimble_debug_live_allocations() <= before
            lib.nimble_debug_fail_allocation(-1)
        # and everything still works afterwards
        splits, lam = B.plan(made, w.traffic, w.eps, 50)
        assert np.array_equal(splits, ref["splits"]) and lam == ref["lam"]
        n_done, lb = B.nimble_plan_solve_adaptive(made, d, w.eps, 200, 10, sp, la)
        assert n_done > 0
    finally:
        lib.nimble_debug_fail_allocation(-1)
        made.close()
    assert lib.nimble_debug_live_allocations() == base


@pytest.mark.parametrize("kind", [0, 1, 2, 3, 4, 5])
def test_grid_barrier_probe(B, kind):
    """The barrier probe behind the benchmark's barrier figures: every design either lets the
    word written before a barrier arrive after it, on every round, or gives up within its
    bounded wait and says so (design 3 releases through a word read at workgroup scope, which
    this part serves from a cache that never sees the release).  A spin limit of zero makes any
    design give up at its first incomplete wait; the kernel still ends normally."""
    import torch
    work = torch.zeros(1 << 19, dtype=torch.uint8, device="cuda:0")
    out = torch.zeros(32, dtype=torch.int32, device="cuda:0")
    print(f"[barrier probe] kind={kind}", flush=True)
    B.nimble_debug_barrier_probe(kind, 1, 256, 25, 1 << 16, work, out)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert o[2:18].sum() > 0 and np.all(o[2:10] == o[2])      # 8 XCDs, evenly filled
    assert np.all(o[10:18] == 0)
    if kind == 3:
        assert o[1] == 1 or (o[0] == 0 and o[18] == 25)
    else:
        assert o[0] == 0 and o[1] == 0 and o[18] == 25
    B.nimble_debug_barrier_probe(kind, 2, 128, 25, 0, work, out)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert o[0] == 0 and (o[1] == 1 or o[18] == 25)
    with pytest.raises(B.NimbleError):
        B.nimble_debug_barrier_probe(7, 1, 256, 5, 10, work, out)
    with pytest.raises(B.NimbleError):
        B.nimble_debug_barrier_probe(0, 1, 256, 5, 10, work[:64], out)


def test_persistent_regime_abandons_cleanly_when_a_barrier_wait_expires(B):
    """With a poll limit of 0 the first incomplete barrier gives up: every workgroup leaves the
    kernel, lambda comes back as NaN, and the topology is usable again afterwards."""
    import math
    w = W.make_config(1)
    h = B.nimble_topo_create(*w.topo.csr())
    try:
        B.nimble_topo_set_regime(h, B.NIMBLE_REGIME_PERSISTENT)
        B.nimble_debug_set_spin_limit(h, 0)
        print("[abandon] spin limit 0", flush=True)
        _, lam = B.plan(h, w.traffic, w.eps, 20)
        assert math.isnan(lam)
        B.nimble_debug_set_spin_limit(h, 1 << 22)
        _, lam = B.plan(h, w.traffic, w.eps, 20)
        assert lam > 0.0
    finally:
        h.close()


@pytest.mark.parametrize("regime,iters", [(0, 1000), (2, 40), (3, 40)])
def test_full_size_config4_against_oracle(oracle_mod, B, regime, iters):
    """Largest configuration, compared element by element: the full 1000 iterations in the
    regime the benchmark times (auto), shortened runs in the others; plus the size-independent
    properties of the result."""
    w = W.make_config(4)
    t = w.topo
    splits, lam = check(oracle_mod, B, t, w.traffic, w.eps, iters, regime=regime)
    np.testing.assert_allclose(np.add.reduceat(splits, t.comm_path_ptr[:-1]), 1.0, rtol=0,
                               atol=1e-12)
    lam2, _ = oracle_mod.congestion(t.n_links, t.cap, t.comm_path_ptr, t.path_link_ptr,
                                    t.path_links, w.traffic, splits)
    assert abs(lam2 - lam) <= 1e-10 * lam
