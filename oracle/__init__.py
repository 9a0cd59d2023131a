"""CPU oracle of the planner -- test infrastructure only.

Nothing in the product path (`paper_2604_00317_amd`) may import this package; only the tests,
`__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` do.
"""
from .oracle import solve, alg1, solve_adaptive, chunked_sum, build, max_threads, set_threads, congestion  # noqa: F401
from .quantize_oracle import quantize  # noqa: F401
