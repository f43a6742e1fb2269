"""Budget arithmetic and FLOPs count: the oracle against the numbers the paper prints, and the
library's host helpers against the oracle (host code only; no GPU involved)."""
import os
import random

import pytest

from oracle import budget_oracle as bo
from paper_2505_22654_amd import binding as vb

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
LLAMA7B = dict(layers=32, d=4096, m=11008)  # see the header of golden/flops_printed.txt


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


FLOPS_ROWS = [(int(r[0]), float(r[1])) for r in _rows("flops_printed.txt")]
# printed rows first, then the rows derived from printed averages (kept in a file of their own)
BUDGET_ROWS = [(int(r[0]), int(r[1]), int(r[2]), float(r[3]), float(r[4]), int(r[5]), int(r[6]),
                float(r[7])) for name in ("budget_printed.txt", "budget_derived.txt")
               for r in _rows(name)]


@pytest.mark.parametrize("n,tflops", FLOPS_ROWS)
def test_oracle_flops_reproduces_printed(n, tflops):
    got = bo.flops([n] * LLAMA7B["layers"], LLAMA7B["d"], LLAMA7B["m"]) / 1e12
    # the paper prints three decimals (some rounded, some cut): within one unit of the last
    assert abs(got - tflops) < 1e-3


def test_oracle_flops_terms_separately():
    # each term alone, from Eq. 6 by hand: one layer, n=2, d=3, m=5
    assert bo.flops([2], 3, 5) == 4 * 2 * 9 + 2 * 4 * 3 + 3 * 2 * 3 * 5
    assert bo.flops([0, 0], 7, 9) == 0
    # quadratic term shows in a stepped schedule: same mean count, more FLOPs
    assert bo.flops([96] * 16 + [32] * 16, 4096, 11008) - bo.flops([64] * 32, 4096, 11008) == \
        2 * 4096 * (16 * 96 * 96 + 16 * 32 * 32 - 32 * 64 * 64)


@pytest.mark.parametrize("n,L,k,r1,r2,n1,n2,avg", BUDGET_ROWS)
def test_oracle_budget_reproduces_printed(n, L, k, r1, r2, n1, n2, avg):
    g1, g2, gavg = bo.budget(n, L, k, r1 / 100, r2 / 100)
    assert (g1, g2) == (n1, n2)
    assert float(gavg) == avg


def test_oracle_solve_r1_printed_example():
    # average 11.1 % at R2 = 33.3 %, pruning at layer 16 of 32 -> R1 = 16.7 % (Sec. 5.1)
    assert round(float(bo.solve_r1(32, 16, 0.111, 0.333)) * 100, 1) == 16.7
    # comparison method pruned to 5.2 % from layer 2 of 32 averages 11.1 % (App. "Remarks on
    # Ensuring Fair Comparisons"): the same formula with r1 = 1
    avg = (2 * 1.0 + 30 * 0.052) / 32
    assert round(avg * 100, 1) == 11.1
    n1, n2, a = bo.budget(1000, 32, 2, 1.0, 0.052)
    assert (n1, n2) == (1000, 52) and round(float(a) / 10, 1) == 11.1


def test_oracle_budget_multi_crop():
    # five crops of 576 tokens at the 11.1 % setting: 480 before the LLM, 160 after, 320 average
    n1, n2, avg = bo.budget(576, 32, 16, 0.167, 0.333)
    assert (5 * n1, 5 * n2, 5 * float(avg)) == (480, 160, 320.0)


# ---- library host helpers against the oracle -------------------------------------------------

@pytest.mark.parametrize("n,tflops", FLOPS_ROWS)
def test_library_flops_matches_oracle(n, tflops):
    want = bo.flops([n] * 32, 4096, 11008)
    got = vb.flops([n] * 32, 4096, 11008)
    assert got == pytest.approx(float(want), rel=1e-14)


def test_library_flops_random_schedules():
    rng = random.Random(7)
    for _ in range(50):
        L = rng.randint(1, 80)
        ns = [rng.randint(0, 20000) for _ in range(L)]
        d, m = rng.randint(1, 9000), rng.randint(1, 30000)
        assert vb.flops(ns, d, m) == pytest.approx(float(bo.flops(ns, d, m)), rel=1e-13)


def test_library_budget_matches_oracle_and_print():
    for n, L, k, r1, r2, n1, n2, avg in BUDGET_ROWS:
        assert vb.budget(n, L, k, r1 / 100, r2 / 100) == (n1, n2, avg)
    rng = random.Random(11)
    for _ in range(200):
        n, L = rng.randint(0, 20000), rng.randint(1, 80)
        k = rng.randint(0, L)
        r1, r2 = rng.random(), rng.random()
        w1, w2, wavg = bo.budget(n, L, k, r1, r2)
        g1, g2, gavg = vb.budget(n, L, k, r1, r2)
        # r * n in binary floating point can land on the other side of a .5 boundary only when
        # the exact product is within rounding of it; the generator does not produce such cases
        assert (g1, g2) == (w1, w2)
        assert gavg == pytest.approx(float(wavg), rel=1e-14)


def test_library_solve_r1():
    assert vb.budget_solve_r1(32, 16, 0.111, 0.333) == pytest.approx(
        float(bo.solve_r1(32, 16, 0.111, 0.333)), rel=1e-14)
    r1 = vb.budget_solve_r1(28, 14, 0.222, 0.333)
    n1, n2, avg = vb.budget(16384, 28, 14, r1, 0.333)
    assert abs(avg / 16384 - 0.222) < 1e-3


def test_library_helper_errors():
    L = vb.lib()
    assert L.vscan_budget(-1, 32, 16, 0.5, 0.5, None, None, None) == vb.VSCAN_ERR_SHAPE
    assert L.vscan_budget(10, 0, 0, 0.5, 0.5, None, None, None) == vb.VSCAN_ERR_SHAPE
    assert L.vscan_budget(10, 4, 5, 0.5, 0.5, None, None, None) == vb.VSCAN_ERR_SHAPE
    assert L.vscan_budget(10, 4, 2, 1.5, 0.5, None, None, None) == vb.VSCAN_ERR_BUDGET
    assert L.vscan_budget(10, 4, 2, float("nan"), 0.5, None, None, None) == vb.VSCAN_ERR_BUDGET
    assert L.vscan_budget(10, 4, 2, 0.5, 0.5, None, None, None) == vb.VSCAN_OK
    assert L.vscan_budget_solve_r1(4, 2, 0.5, 0.5, None) == vb.VSCAN_ERR_NULL
    with pytest.raises(vb.VscanError):
        vb.budget_solve_r1(32, 16, 0.9, 0.333)  # would need r1 > 1
    with pytest.raises(vb.VscanError):
        vb.budget_solve_r1(32, 0, 0.5, 0.0)     # zero denominator
    assert L.vscan_flops(None, 1, 1, 1, None) == vb.VSCAN_ERR_NULL
    with pytest.raises(vb.VscanError):
        vb.flops([1, -1], 8, 8)
    with pytest.raises(vb.VscanError):
        vb.flops([1], 0, 8)
