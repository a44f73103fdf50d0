"""Analytical cost model of the paper, in exact fractions -- TEST INFRASTRUCTURE.

The per-GPU expected costs of one sequence embedding table in one training iteration under the
four uniform strategies (Section 3.2: the six metrics; the memory-cost table and the
communication-cost table).  Written out cell by cell from those two tables with
fractions.Fraction, so nothing is rounded; "N/A" cells are 0.  Only tests/ may import this.

Pins (tests/test_oracle_cost_model.py): the activation sizes the paper prints for its models, the
break-even probabilities that follow from the tables (memory (6 - 1/U)/B, traffic 1/(6B) at
all-reduce = 3 x all-to-all bandwidth), and the all-to-all reductions the paper measured against
the coverage it predicted.
"""
from fractions import Fraction as Fr

RW, CW, DP, FLEX = 0, 1, 2, 3
STATIC_MEMORY, INPUT_DIST, ROWS_ACCESSED, DYNAMIC_MEMORY, DYNAMIC_COMM, STATIC_COMM = range(6)


def cost_model(p: dict, strategy: int):
    """p: E, D, dtype_bytes, L, W, N, B, a2a_global, a2a_intra, ar_global, ar_cross, dp_multiplier.
    Returns the six metrics as Fractions (bytes, ids, row elements, bytes, seconds, seconds)."""
    f = {k: Fr(v) for k, v in p.items()}
    E, D, s, L, W, N, B = f["E"], f["D"], f["dtype_bytes"], f["L"], f["W"], f["N"], f["B"]
    U = N * W
    six = f["dp_multiplier"]
    if strategy == RW:
        return [E / U * D * s, B * L, U * B * (L / U) * D, 2 * B * L * D * s, B * L * D * s / f["a2a_global"], Fr(0)]
    if strategy == CW:
        return [E * (D / U) * s, U * B * L, U * B * L * (D / U), 2 * B * L * D * s, B * L * D * s / f["a2a_global"], Fr(0)]
    if strategy == DP:
        return [six * E * D * s, Fr(0), B * L * D, B * L * D * s, Fr(0), E * D * s / f["ar_global"]]
    if strategy == FLEX:
        return [six * (E / W) * D * s, B * L, W * B * (L / W) * D, 2 * B * L * D * s, B * L * D * s / f["a2a_intra"],
                (E / W) * D * s / f["ar_cross"]]
    raise ValueError(strategy)


def tier_traffic(tier_counts, D: int, dtype_bytes: int):
    """Row bytes that cross GPUs in one direction of one pass, from the lookups per tier
    (replicated, group, sharded): [all sharded, global all-to-all left, intra-group all-to-all,
    share of the global all-to-all avoided]."""
    t0, t1, t2 = (Fr(int(x)) for x in tier_counts)
    n = t0 + t1 + t2
    row = Fr(D) * dtype_bytes
    return [n * row, t2 * row, t1 * row, (t0 + t1) / n if n else Fr(0)]
