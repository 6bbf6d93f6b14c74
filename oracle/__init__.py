"""CPU oracle for the fused communication + GEMM hot path (test infrastructure only).

Plain, slow, fp64 numpy/Python statements of what AllGather-GEMM, GEMM-ReduceScatter,
GEMM + AllReduce and MoE AllGather + grouped GEMM compute, and of the integer tile schedules and routing
tables that go with them.  Written from the paper's definitions; shares no code with the
HIP library and never imports it.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the product path must not.

Parity pins (tests/test_oracle_*.py): brute-force loops on tiny inputs, closed forms,
library special cases (torch dtype conversion, numpy stable argsort / bincount), the
paper's worked tiling example, bijection / conservation invariants.
Unpinned against the paper: the helper semantics of the MoE tile schedule (stage of a
tile, bisect helper), whose bodies the paper does not print -- pinned by invariants only.
"""
from . import formats, ag_gemm, gemm_rs, gemm_ar, moe, schedule, compare  # noqa: F401
