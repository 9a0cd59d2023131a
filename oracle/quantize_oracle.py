"""CPU oracle for the plan post-processing policies: TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU leg may import this file; the product
never does, and the two share no code.

What it computes.  The planner's split fractions have to become what the dataplane consumes:
per pair, a list of paths with a byte amount each (the Paths / Flows lists of Algorithm 1), in
whole chunks so that messages are not fragmented below the chunk granularity, and with small
messages kept off the multi-hop paths (Sec. V-A: forwarding is switched off for messages of
1 MB or less; the introduction's "size threshold that prevents excessive fragmentation of
small messages").  For a pair with demand d bytes and candidate counts c_j (times candidate j
was chosen in T iterations, so split_j = c_j / T):

  * d <= theta (the small-message threshold): everything on candidate 0, the direct or
    fewest-relay path.
  * otherwise N = floor(d / chi) whole chunks and a residual res = d - N * chi < chi.
    Candidate j gets q_j = floor(N * c_j / T) chunks; the R = N - sum_j q_j chunks that are left
    (R < number of candidates) go, one each, to the candidates with the largest remainders
    N * c_j mod T (largest-remainder apportionment; ties to the lower index).  The residual
    bytes, which Algorithm 1 routes as one last flow, go to the candidate with the largest
    count (ties to the lower index).
    flow_j = chi * (q_j + extra_j) + (res if j is that candidate else 0).

Readings (the paper names the policies but gives no rule): largest remainder for the chunk
apportionment, the most-used candidate for the residual, candidate 0 for small messages.

All arithmetic on chunk numbers is exact integer arithmetic; the byte amounts are exact in
binary64 for integer demands below 2^53.

Pins (tests/test_quantize_pins.py): a hand-worked apportionment, conservation, the
one-chunk bound |flow_j - d*c_j/T| < chi (+ res for the residual's candidate), whole chunks,
the quota property floor/ceil, small messages on candidate 0, chi = 1 and T | N reproduce the
exact shares, and invariance of every pair's result to the other pairs.
"""
from __future__ import annotations

import numpy as np


def quantize(comm_path_ptr, demand, splits, iters, chi, theta):
    """Returns flows [n_paths] in bytes (float64)."""
    cp = np.asarray(comm_path_ptr, dtype=np.int64)
    d = np.asarray(demand, dtype=np.float64)
    x = np.asarray(splits, dtype=np.float64)
    T = int(iters)
    chi_i = int(chi)
    assert chi_i >= 1 and chi_i == chi and T >= 1
    flows = np.zeros(int(cp[-1]), dtype=np.float64)
    for k in range(len(cp) - 1):
        a, b = int(cp[k]), int(cp[k + 1])
        n = b - a
        if n == 0:
            continue
        dk = float(d[k])
        if dk <= theta:
            flows[a] = dk
            continue
        c = [int(round(float(x[a + j]) * T)) for j in range(n)]
        N = int(np.floor(dk / chi_i))
        res = dk - float(N * chi_i)
        q = [(N * c[j]) // T for j in range(n)]
        rem = [(N * c[j]) % T for j in range(n)]
        R = N - sum(q)
        order = sorted(range(n), key=lambda j: (-rem[j], j))
        extra = [0] * n
        for j in order[:R]:
            extra[j] = 1
        jmax = max(range(n), key=lambda j: (c[j], -j))
        for j in range(n):
            f = float(chi_i * (q[j] + extra[j]))
            if j == jmax:
                f = f + res
            flows[a + j] = f
    return flows
