"""The host-side layout code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU).

csrc/host_topo.cpp -- validation, reverse CSR, octets / tiles / strips / link blocks, forward
records in all their formats -- is index arithmetic over vectors.  It is compiled here with g++
-fsanitize=address,undefined (no HIP involved) together with a small driver that runs every
host-only helper on a topology and checks the round trips, over the benchmark fabrics, ragged
random topologies and the layout options that reach the other code paths.  Any out-of-bounds
access, overflow or misaligned access ends the driver with a non-zero status.
"""
import os
import subprocess

import numpy as np
import pytest

from paper_2604_00317_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = tmp_path_factory.mktemp("asan") / "host_layout_driver"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-static-libubsan",
           "-o", str(out), os.path.join(ROOT, "tests", "host_layout_driver.cpp"),
           os.path.join(ROOT, "paper_2604_00317_amd", "csrc", "host_topo.cpp")]
    subprocess.run(cmd, check=True)
    return str(out)


def _dump(t, d):
    os.makedirs(d, exist_ok=True)
    np.asarray(t.cap, dtype=np.float64).tofile(os.path.join(d, "cap.bin"))
    np.asarray(t.comm_path_ptr, dtype=np.int32).tofile(os.path.join(d, "cp.bin"))
    np.asarray(t.path_link_ptr, dtype=np.int32).tofile(os.path.join(d, "lp.bin"))
    np.asarray(t.path_links, dtype=np.int32).tofile(os.path.join(d, "pl.bin"))


def _topologies():
    rng = np.random.default_rng(2024)
    yield "config0", W.config_topology(0)
    yield "config1", W.config_topology(1)
    yield "config3", W.config_topology(3)
    yield "product24x8", W.build_fabric(24, 8, 8, [[r, r ^ 1] for r in range(8)])
    yield "mesh35", W.two_candidate_mesh(35)
    for i, (E, K, pm, lm) in enumerate(((7, 3, 4, 3), (40, 130, 9, 5), (300, 1000, 20, 6),
                                        (64, 65, 33, 4), (90, 17, 100, 7), (1, 5, 1, 1),
                                        (500, 3000, 12, 2), (50, 40, 127, 2), (30, 200, 64, 1),
                                        (120, 900, 40, 2), (70000, 300, 12, 2))):
        yield f"random{i}", W.random_topology(rng, E, K, pm, lm)


ENVS = {
    "default": {},
    "tiles-1": {"NIMBLE_TUNE_TILES": "1", "NIMBLE_TUNE_TILE_MIN_ITEMS": "1"},
    "tiles-24-dense": {"NIMBLE_TUNE_TILES": "1", "NIMBLE_TUNE_TILE_MIN_ITEMS": "24",
                       "NIMBLE_TUNE_TILES_DENSE_ONLY": "1"},
    "dictionary": {"NIMBLE_TUNE_RECORD_DICT": "1"},
    "record-major": {"NIMBLE_TUNE_RECORD_LANE_MAJOR": "0"},
    "table32-blocks-of-one-pass": {"NIMBLE_TUNE_RECORD_TABLE16": "0",
                                   "NIMBLE_TUNE_BLOCK_PASSES": "1"},
}


@pytest.mark.parametrize("env_name", list(ENVS))
def test_host_layouts_under_sanitizers(driver, tmp_path, env_name):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1", **ENVS[env_name])
    for name, t in _topologies():
        if name == "product24x8" and env_name not in ("default", "dictionary"):
            continue                      # (the large one only where its size matters)
        d = str(tmp_path / name)
        _dump(t, d)
        r = subprocess.run([driver, d], env=env, capture_output=True, text=True)
        assert r.returncode == 0, (name, env_name, r.stdout[-300:], r.stderr[-2000:])
        assert r.stdout.startswith("OK"), (name, r.stdout)
