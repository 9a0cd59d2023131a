"""The pins must notice plausible single-line mistakes in the oracles (no GPU needed).

Every entry below alters one statement of a COPY of an oracle source (the tracked files are
never touched), builds it into a temporary directory and runs the pin file of that oracle
against the altered library in a child process: the pins have to fail.  The list covers the
statements of the method one by one -- tie rule, step normalisation, price definition in both
cost modes, load and congestion bookkeeping, width, the adaptive step and its bound, and
Algorithm 1's cost, schedule and chunk rule.  A last case runs the adaptive oracle with a plain
sequential sum in place of the chunked one and checks that the stop iteration is the same.
"""
import json
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle")
SOURCES = ["nimble_oracle.c", "alg1_oracle.c", "adaptive_oracle.c"]

# (source file, statement, altered statement, pin file that must fail)
MUTATIONS = [
    # --- fixed-step method -------------------------------------------------------------------
    ("nimble_oracle.c", "if (c < cbest)", "if (c <= cbest)", "test_oracle_pins.py"),
    ("nimble_oracle.c", "double g = u * invrho;", "double g = u;", "test_oracle_pins.py"),
    ("nimble_oracle.c", "double t2 = 1.0 + t1;", "double t2 = 1.0 + t1 + t1;",
     "test_oracle_pins.py"),
    # sum mode priced without the capacity
    ("nimble_oracle.c", "price[e] = use_max ? len[e] : len[e] * invcap[e];\n        S[e] = 0.0;",
     "price[e] = len[e];\n        S[e] = 0.0;", "test_oracle_pins.py"),
    ("nimble_oracle.c", "price[e] = use_max ? len[e] : len[e] * invcap[e];\n        }",
     "price[e] = len[e];\n        }", "test_oracle_pins.py"),
    # bottleneck mode priced WITH the capacity (initial prices, then the update)
    ("nimble_oracle.c", "price[e] = use_max ? len[e] : len[e] * invcap[e];\n        S[e] = 0.0;",
     "price[e] = len[e] * invcap[e];\n        S[e] = 0.0;", "test_oracle_pins.py"),
    ("nimble_oracle.c", "price[e] = use_max ? len[e] : len[e] * invcap[e];\n        }",
     "price[e] = len[e] * invcap[e];\n        }", "test_oracle_pins.py"),
    ("nimble_oracle.c", "double u = load[e] * invcap[e];", "double u = load[e];",
     "test_oracle_pins.py"),
    ("nimble_oracle.c", "S[e] = S[e] + u;", "S[e] = u;", "test_oracle_pins.py"),
    ("nimble_oracle.c", "*lambda = smax / T;", "*lambda = smax;", "test_oracle_pins.py"),
    ("nimble_oracle.c", "c = c + pe;", "c = pe;", "test_oracle_pins.py"),
    ("nimble_oracle.c", "if (pe > c) c = pe;", "c = c + pe;", "test_oracle_pins.py"),
    ("nimble_oracle.c", "if (stamp[e] != k) {", "if (1) {", "test_oracle_pins.py"),
    ("nimble_oracle.c", "const int p = comm_path_ptr[k] + choice[k];",
     "const int p = comm_path_ptr[k];", "test_oracle_pins.py"),
    ("nimble_oracle.c", "if (w > rho) rho = w;", "if (w < rho || rho == 0.0) rho = w;",
     "test_oracle_pins.py"),
    ("nimble_oracle.c", "load[e] = load[e] + demand[k];", "load[e] = load[e] + 1.0;",
     "test_oracle_pins.py"),
    ("nimble_oracle.c", "len[e] = len_io ? len_io[e] : 1.0;", "len[e] = 1.0;",
     "test_oracle_pins.py"),
    # --- adaptive step -----------------------------------------------------------------------
    ("adaptive_oracle.c", "price[e] = use_max ? len[e] : len[e] * invcap[e];",
     "price[e] = len[e] * invcap[e];", "test_adaptive_pins.py"),
    ("adaptive_oracle.c", "price[e] = use_max ? 1.0 : invcap[e];", "price[e] = invcap[e];",
     "test_adaptive_pins.py"),
    ("adaptive_oracle.c", "price[e] = use_max ? len[e] : len[e] * invcap[e];",
     "price[e] = len[e];", "test_adaptive_pins.py"),
    ("adaptive_oracle.c", "const double su = sigma * u[e];", "const double su = u[e];",
     "test_adaptive_pins.py"),
    ("adaptive_oracle.c", "const double sigma = 1.0 / umax;", "const double sigma = umax;",
     "test_adaptive_pins.py"),
    ("adaptive_oracle.c", "weight[p] = weight[p] + sigma;", "weight[p] = weight[p] + 1.0;",
     "test_adaptive_pins.py"),
    ("adaptive_oracle.c", "lb_t = alpha / D;", "lb_t = alpha;", "test_adaptive_pins.py"),
    ("adaptive_oracle.c", "if (lam <= bound) break;", "if (lam <= bound * 4.0) break;",
     "test_adaptive_pins.py"),
    ("adaptive_oracle.c", "if (c < cbest) {", "if (c <= cbest) {", "test_adaptive_pins.py"),
]


def _alg1_mutations():
    cands = [
        ("if (cp < c_best) {", "if (cp <= c_best) {"),           # tie rule of the scan
        ("if (ce > cp) cp = ce;", "cp = cp + ce;"),                # additive instead of bottleneck
        ("c[e] = L[e] * invcap[e];", "c[e] = L[e];"),              # cost without the capacity
        ("c[e] = L[e] * invcap[e];", ";"),                         # costs never updated
        ("const double want = r[k] * phi;", "const double want = r[k];"),
        ("if (!(f > 0.0)) f = chi;", ";"),                         # the one-chunk rule
        ("r[k] = r[k] - f;", "r[k] = 0.0;"),
        ("L[e] = L[e] + f;", "L[e] = f;"),
    ]
    return [("alg1_oracle.c", a, b, "test_alg1_pins.py") for a, b in cands]


def _build_variant(tmpdir, tag, fname, old, new):
    texts = {f: open(os.path.join(ORACLE, f)).read() for f in SOURCES}
    assert texts[fname].count(old) >= 1, f"statement not found in {fname}: {old!r}"
    texts[fname] = texts[fname].replace(old, new, 1)
    d = os.path.join(tmpdir, tag)
    os.makedirs(d)
    paths = []
    for f, text in texts.items():
        paths.append(os.path.join(d, f))
        with open(paths[-1], "w") as out:
            out.write(text)
    lib = os.path.join(d, "libvariant.so")
    subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
                    "-o", lib, *paths, "-lm"], check=True)
    return lib


def _pins_fail(lib, pin_file):
    env = dict(os.environ, NIMBLE_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", pin_file),
                        "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env,
                       capture_output=True, text=True)
    return r.returncode != 0, r.stdout[-400:]


def test_every_listed_mistake_fails_a_pin(tmp_path):
    muts = MUTATIONS + _alg1_mutations()

    def one(i):
        fname, old, new, pins = muts[i]
        lib = _build_variant(str(tmp_path), f"m{i}", fname, old, new)
        return _pins_fail(lib, pins)

    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(one, range(len(muts))))
    missed = [muts[i][:3] for i, (failed, _) in enumerate(results) if not failed]
    assert not missed, f"mutations that no pin notices: {missed}"


def test_unaltered_copy_passes(tmp_path):
    """The harness itself: an unchanged copy built the same way passes the same pin files."""
    lib = _build_variant(str(tmp_path), "same", "nimble_oracle.c", "if (c < cbest)",
                         "if (c < cbest)")
    for pins in ("test_oracle_pins.py", "test_adaptive_pins.py", "test_alg1_pins.py"):
        failed, tail = _pins_fail(lib, pins)
        assert not failed, tail


_STOP_SCRIPT = r"""
import json, sys
import oracle
from paper_2604_00317_amd import workloads as W
out = {}
for cfg in (0, 1, 3):
    w = W.make_config(cfg)
    r = oracle.solve_adaptive(*w.topo.csr(), w.traffic, w.eps, 20000, 10)
    out[str(cfg)] = [r["iters"], r["lam"], r["lb"]]
print(json.dumps(out))
"""


def test_stop_iteration_does_not_depend_on_the_sum_association(tmp_path):
    """The adaptive oracle adds the two sums of its lower bound in chunks of 256 terms.  With a
    plain left-to-right sum instead the bound moves by rounding only: the solve must stop at the
    same iteration on the benchmark fabrics, with the same lambda (the plan does not depend on
    the bound) and a bound equal to 1e-12."""
    lib = _build_variant(str(tmp_path), "seq", "adaptive_oracle.c", "#define ADAPTIVE_CHUNK 256",
                         "#define ADAPTIVE_CHUNK (1 << 30)")
    res = {}
    for tag, env in (("chunked", dict(os.environ)),
                     ("sequential", dict(os.environ, NIMBLE_ORACLE_LIB=lib))):
        env.pop("NIMBLE_ORACLE_LIB", None) if tag == "chunked" else None
        r = subprocess.run([sys.executable, "-c", _STOP_SCRIPT], cwd=ROOT, env=env,
                           capture_output=True, text=True, check=True)
        res[tag] = json.loads(r.stdout.strip().splitlines()[-1])
    for cfg in ("0", "1", "3"):
        a, b = res["chunked"][cfg], res["sequential"][cfg]
        assert a[0] == b[0], f"config {cfg}: stop iteration {a[0]} vs {b[0]}"
        assert a[1] == b[1]
        assert b[2] == pytest.approx(a[2], rel=1e-12)
