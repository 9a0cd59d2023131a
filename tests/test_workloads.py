"""The synthetic input generators produce the shapes the benchmark configurations name."""
import numpy as np
import pytest

from paper_2604_00317_amd import workloads as W

SHAPES = {0: (56, 392, 728, 56), 1: (240, 2832, 11184, 152), 3: (16256, 252032, 1179008, 2112)}


@pytest.mark.parametrize("cfg", [0, 1, 3])
def test_config_shapes(cfg):
    t = W.config_topology(cfg)
    assert (t.n_comm, t.n_paths, t.nnz, t.n_links) == SHAPES[cfg]
    assert t.comm_path_ptr[0] == 0 and t.comm_path_ptr[-1] == t.n_paths
    assert np.all(np.diff(t.comm_path_ptr) > 0) and np.all(np.diff(t.path_link_ptr) > 0)
    assert t.path_links.min() >= 0 and t.path_links.max() == t.n_links - 1
    # every link is used and no path repeats a link
    assert np.unique(t.path_links).size == t.n_links
    lens = np.diff(t.path_link_ptr)
    assert lens.max() <= 5
    for p in np.random.default_rng(0).integers(0, t.n_paths, 200):
        seg = t.path_links[t.path_link_ptr[p]:t.path_link_ptr[p + 1]]
        assert np.unique(seg).size == seg.size


def test_path_order_direct_first_then_relays():
    t = W.build_fabric(1, 4)
    # commodity 0 is GPU0 -> GPU1: direct link id 0, relays via GPU2 then GPU3
    assert t.path_links[t.path_link_ptr[0]:t.path_link_ptr[1]].tolist() == [0]
    via2 = t.path_links[t.path_link_ptr[1]:t.path_link_ptr[2]].tolist()
    via3 = t.path_links[t.path_link_ptr[2]:t.path_link_ptr[3]].tolist()
    assert via2 == [1, 2 * 3 + 1] and via3 == [2, 3 * 3 + 1]


def test_inter_node_paths_are_rail_matched():
    t = W.build_fabric(2, 8, 4, W.pair_access(4))
    k = int(np.nonzero((t.src == 0) & (t.dst == 8))[0][0])
    assert t.comm_path_ptr[k + 1] - t.comm_path_ptr[k] == 16
    n_intra = 2 * 56
    for p in range(t.comm_path_ptr[k], t.comm_path_ptr[k + 1]):
        seg = t.path_links[t.path_link_ptr[p]:t.path_link_ptr[p + 1]]
        nic = seg[seg >= n_intra]
        assert nic.size == 3                      # GPU->NIC, NIC->NIC, NIC->GPU
        assert np.all(t.cap[nic] == W.NIC_CAP)
        assert 3 <= seg.size <= 5


def test_traffic_is_integral_seeded_and_skewed():
    w0 = W.make_config(0)
    assert np.all(w0.traffic == np.floor(w0.traffic))
    assert np.all(w0.traffic.reshape(8, 7).sum(axis=1) == float(1 << 26))
    w1a, w1b = W.make_config(1), W.make_config(1)
    assert np.array_equal(w1a.traffic, w1b.traffic)
    assert np.all(w1a.traffic % (4096 * 2) == 0)
    # tokens*top_k routed slots per source, minus the local share
    per_src = w1a.traffic.reshape(16, 15).sum(axis=1) / (4096 * 2)
    assert np.all(per_src <= 4096 * 2) and np.all(per_src > 0.5 * 4096 * 2)
    assert w1a.traffic.max() > 4 * np.median(w1a.traffic)
    b = W.make_config(2, batch=3)
    assert b.traffic.shape == (3, 56) and not np.array_equal(b.traffic[0], b.traffic[1])


def test_inclusion_probabilities_sum_to_k():
    w = np.arange(1, 65, dtype=np.float64) ** -1.6
    pi = W._inclusion_probabilities(w, 8)
    assert pi.sum() == pytest.approx(8.0) and pi.max() <= 1.0 + 1e-15 and pi.min() > 0
