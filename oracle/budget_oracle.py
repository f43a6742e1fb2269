"""Oracle for the host-side budget arithmetic: stage budgets and the theoretical FLOPs count.

Test infrastructure only: nothing in the product path imports this module.

Written out from the definitions in exact arithmetic (fractions / Python integers):
  * Sec. 5.1 "Implementation Details" and App. "Remarks on Ensuring Fair Comparisons": with
    `prune_layer` of `n_layers` decoder layers seeing n1 = round(r1 * n) tokens and the remaining
    layers n2 = round(r2 * n1), the layer-averaged count is
    (prune_layer * n1 + (n_layers - prune_layer) * n2) / n_layers.
  * Eq. 6 (App. "Computational Complexity"): sum over layers of 4 n d^2 + 2 n^2 d + 3 n d m.
Pinned by the numbers the paper prints (tests/golden/).
"""
from fractions import Fraction
from typing import Sequence, Tuple


def _nearest(v: Fraction) -> int:
    """Nearest integer, halves up (v >= 0)."""
    return int((v + Fraction(1, 2)).__floor__())


def budget(n_visual: int, n_layers: int, prune_layer: int, r1: float, r2: float
           ) -> Tuple[int, int, Fraction]:
    n1 = _nearest(Fraction(r1) * n_visual)
    n2 = _nearest(Fraction(r2) * n1)
    avg = Fraction(prune_layer * n1 + (n_layers - prune_layer) * n2, n_layers)
    return n1, n2, avg


def solve_r1(n_layers: int, prune_layer: int, avg_rate: float, r2: float) -> Fraction:
    """r1 with (prune_layer * r1 + (n_layers - prune_layer) * r1 * r2) / n_layers == avg_rate."""
    return Fraction(avg_rate) * n_layers / (prune_layer + (n_layers - prune_layer) * Fraction(r2))


def flops(n_per_layer: Sequence[int], d: int, m: int) -> int:
    total = 0
    for n in n_per_layer:
        total += 4 * n * d * d + 2 * n * n * d + 3 * n * d * m
    return total
