"""CPU oracle for the fused communication + GEMM hot path (test infrastructure only).

Plain, slow, fp64 numpy/Python statements of what AllGather-GEMM, GEMM-ReduceScatter,
GEMM + AllReduce and MoE AllGather + grouped GEMM compute, and of the integer tile schedules and routing
tables that go with them.  Written from the paper's definitions; shares no code with the
HIP library and never imports it.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the product path must not.

Parity pins (tests/test_oracle_*.py): brute-force loops on tiny inputs, closed forms,
library special cases (torch dtype conversion, numpy stable argsort / bincount), the
paper's worked tiling example, bijection / conservation invariants, multi-node visiting orders
worked by hand from the two swizzle listings (tests/golden/multinode_order_three_nodes.txt) and
re-derived from the ownership rule of shared tile rows, the MoE tile stage tied to the producer's
delivery order (ag_gemm.arrival_order) with hand-worked orders for 3 and 4 ranks.
The bodies of the MoE schedule's helpers (stage of a tile, bisect) are not printed in the paper:
the stage is read as the delivery position of the last shard a tile needs and the bisect as
"entries <= x"; both readings are pinned by re-deriving every tile's source ranks from gather_idx.
"""
from . import formats, ag_gemm, gemm_rs, gemm_ar, moe, moe_rs, schedule, compare  # noqa: F401
