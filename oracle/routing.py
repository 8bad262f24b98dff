"""Routing-decision oracle (test infrastructure only): the paper's score (section 3), the two phases of its
routing algorithm (section 5) and the discretisation of the appendix "Decision-Engine Discretization", written
out plainly in Python.  Independent of the library's C implementation."""
import math

QPS_LEVELS = (0.5, 1, 2, 4, 6, 8, 10, 12, 16, 20)       # the benchmark levels of the offline phase


def score(w_ttft, w_tpot, delta_ttft, delta_tpot):
    """Benefit of local processing: weighted relative TTFT improvement minus weighted relative TPOT degradation."""
    return w_ttft * delta_ttft - w_tpot * delta_tpot


def build_table(delta_ttft, delta_tpot, w_ttft, w_tpot):
    """Offline phase: per cell, 1 if the score is positive."""
    return [1 if score(w_ttft, w_tpot, a, b) > 0 else 0 for a, b in zip(delta_ttft, delta_tpot)]


def cell(ratio_centers, n_in, n_out, n_ctx, qps):
    ctx = 0 if n_ctx <= 512 else (1 if n_ctx <= 4096 else 2)      # small / large / huge
    ratio = n_in / n_out
    r = min(range(9), key=lambda i: abs(math.log(ratio) - math.log(ratio_centers[i])))
    q = min(range(10), key=lambda i: abs(QPS_LEVELS[i] - qps))
    return (ctx * 9 + r) * 10 + q


def decide(table, ratio_centers, turn, n_in, n_out, n_ctx, qps):
    """Online phase: turn 1 has no cached KV and always takes the prefill-node path."""
    if turn == 1:
        return 0
    return table[cell(ratio_centers, n_in, n_out, n_ctx, qps)]
