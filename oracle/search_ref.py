"""Plain-Python oracle of the layer-wise bitwidth search (Sec. III-C, Eq. 3, Eq. 4, Alg. 1).
TEST INFRASTRUCTURE ONLY: nothing in the HIP library imports this file and this file imports
nothing from it.

The search is a heuristic, so the oracle is the algorithm's steps in the paper's order.  Inputs are
tables, not a model: lat[l][wi][ai] is the latency of layer l with weights at level wi and
activations at level ai, rmse_w[l][wi] / rmse_a[l][ai] the quantization error (Eq. 2) of the
layer's weight tensor / input activation tensor at that level.  Levels are indices into
LEVELS = (8, 4, 2) bits (Sec. III-C: the widths the search chooses from).

Readings taken where the text leaves a choice (each is also listed in the design notes):
  * RMSE_i(a, w) of a layer is the sum of its weight tensor's and its activation tensor's error.
  * Layer-wise metrics are those of the current assignment (W, A), not of the assignment after
    the next degradation.
  * Candidates are the layers that can still be lowered (W or A above 2 bits); ranking takes the
    first k of them, ties going to the lower layer index, and the re-ranking is stable as well.
  * "Degrade" lowers by one level (8 -> 4 -> 2); a layer already at 2 bits in the table being
    lowered is passed over.
  * Speedup strategy (Eq. 3): ratio = total latency at (8, 8) / total latency now; the search ends
    as soon as ratio >= alpha, or when nothing can be lowered any more (constraint not met).
  * RMSE strategy (Eq. 4): ratio = total error now / total error at (8, 8); the bound is a budget:
    the first degradation that takes the ratio above beta is taken back and ends the search, so the
    result always satisfies Eq. 4.
  * Totals are summed over the layers in index order, in float64.

Pins (tests/test_oracle_search.py): two hand-traced runs per strategy, the reduction to a plain
greedy descent for k = 1, exhaustive check of the constraints on random tables.
Unpinned: nothing in this file.
"""
from __future__ import annotations

LEVELS = (8, 4, 2)
LOWEST = len(LEVELS) - 1


def total_latency(lat, wi, ai) -> float:
    """Left side of Eq. 3 / objective of Eq. 4."""
    t = 0.0
    for l in range(len(wi)):
        t += lat[l][wi[l]][ai[l]]
    return t


def layer_rmse(rmse_w, rmse_a, l, wi, ai) -> float:
    return rmse_w[l][wi[l]] + rmse_a[l][ai[l]]


def total_rmse(rmse_w, rmse_a, wi, ai) -> float:
    """Objective of Eq. 3 / left side of Eq. 4."""
    t = 0.0
    for l in range(len(wi)):
        t += layer_rmse(rmse_w, rmse_a, l, wi, ai)
    return t


def search(lat, rmse_w, rmse_a, strategy: str, constraint: float, k: int):
    """Alg. 1.  Returns (w_bits, a_bits, ratio, met): the bit widths per layer, the final ratio and
    whether the constraint holds at the end."""
    if strategy not in ("speedup", "rmse"):
        raise ValueError("strategy is 'speedup' or 'rmse'")
    n = len(lat)
    if k < 1:
        raise ValueError("k >= 1")
    wi, ai = [0] * n, [0] * n                                   # W, A <- (8, ..., 8)

    def current_ratio():
        if strategy == "speedup":
            return base / total_latency(lat, wi, ai)
        return total_rmse(rmse_w, rmse_a, wi, ai) / base

    base = total_latency(lat, wi, ai) if strategy == "speedup" else total_rmse(rmse_w, rmse_a, wi, ai)
    if not base > 0.0:
        raise ValueError("the (8, 8) total must be positive")
    ratio = 1.0
    done = strategy == "speedup" and ratio >= constraint
    while not done:
        cand = [l for l in range(n) if wi[l] < LOWEST or ai[l] < LOWEST]
        if not cand:
            break
        lat_l = {l: lat[l][wi[l]][ai[l]] for l in cand}        # Layerwise_metric
        err_l = {l: layer_rmse(rmse_w, rmse_a, l, wi, ai) for l in cand}
        if strategy == "speedup":
            top = sorted(cand, key=lambda l: (-lat_l[l], l))[:k]        # Lat_rank: the k slowest
            order = sorted(top, key=lambda l: (err_l[l], l))            # RMSE_rerank: least error first
        else:
            top = sorted(cand, key=lambda l: (err_l[l], l))[:k]         # RMSE_rank: the k with least error
            order = sorted(top, key=lambda l: (-lat_l[l], l))           # Lat_rerank: slowest first
        for table in (wi, ai):                                  # Degrade_level(list, W), then (list, A)
            for l in order:
                if table[l] == LOWEST:
                    continue
                table[l] += 1
                r = current_ratio()
                if strategy == "speedup":
                    ratio = r
                    if ratio >= constraint:
                        done = True
                        break
                else:
                    if r > constraint:
                        table[l] -= 1                           # over the budget: take it back and stop
                        done = True
                        break
                    ratio = r
            if done:
                break
    met = ratio >= constraint if strategy == "speedup" else ratio <= constraint
    return [LEVELS[i] for i in wi], [LEVELS[i] for i in ai], ratio, met
