"""The comparison rules of tests/parity_utils.py, checked on the CPU with planted mistakes: a
rule that accepts a wrong selection (or rejects a right one) would void the GPU parity tests
that rely on it.  Oracle side only; no GPU, no HIP library."""
import dataclasses

import numpy as np
import pytest

from oracle import vscan_oracle as vo
from paper_2505_22654_amd import workloads as wl
from tests import parity_utils as pu


def test_valid_topk_accepts_the_top_set_and_rejects_planted_mistakes():
    s = np.array([0.30, 0.05, 0.20, 0.10, 0.25, 0.10])
    pool = np.arange(6)
    pu.assert_valid_topk([0, 2, 4], pool, s, 3, "top-3")
    with pytest.raises(AssertionError):      # a clearly worse token kept
        pu.assert_valid_topk([0, 1, 4], pool, s, 3, "worse")
    with pytest.raises(AssertionError):      # wrong count
        pu.assert_valid_topk([0, 4], pool, s, 3, "count")
    with pytest.raises(AssertionError):      # duplicate
        pu.assert_valid_topk([0, 0, 4], pool, s, 3, "dup")
    with pytest.raises(AssertionError):      # outside the candidate pool
        pu.assert_valid_topk([0, 2, 4], np.array([0, 1, 2, 3]), s, 3, "pool")
    # exact tie at the boundary (tokens 3 and 5 both 0.10): the lower index must win
    pu.assert_valid_topk([0, 2, 3, 4], pool, s, 4, "tie-low")
    with pytest.raises(AssertionError):
        pu.assert_valid_topk([0, 2, 4, 5], pool, s, 4, "tie-high")


def test_valid_topk_tolerates_only_gaps_inside_the_score_tolerance():
    s = np.array([0.5, 0.2, 0.2 * (1 - 0.5 * pu.SCORE_RTOL), 0.1])
    pool = np.arange(4)
    pu.assert_valid_topk([0, 1], pool, s, 2, "oracle's own")
    pu.assert_valid_topk([0, 2], pool, s, 2, "inside the tolerance")     # fp32 cannot tell them apart
    s[2] = 0.2 * (1 - 4 * pu.SCORE_RTOL)
    with pytest.raises(AssertionError):
        pu.assert_valid_topk([0, 2], pool, s, 2, "outside the tolerance")


def test_topk_rows_demand_identity_where_the_margin_clears():
    s = np.array([[0.4, 0.3, 0.2, 0.1]])
    ref = vo.topk(s, 2)
    assert pu.check_topk_rows(ref.copy(), ref, s, 2, "same") == 0
    with pytest.raises(AssertionError):
        pu.check_topk_rows(np.array([[0, 2]], np.int32), ref, s, 2, "clear boundary")
    near = np.array([[0.4, 0.3, 0.3 * (1 - 0.5 * pu.SCORE_RTOL), 0.1]])
    ref = vo.topk(near, 2)
    assert ref.tolist() == [[0, 1]]
    assert pu.check_topk_rows(np.array([[0, 2]], np.int32), ref, near, 2, "near tie") == 1
    with pytest.raises(AssertionError):      # descending output is never valid
        pu.check_topk_rows(np.array([[2, 0]], np.int32), ref, near, 2, "order")


def _enc_case():
    shape = wl.EncoderShape(dtype=wl.F32, batch=1, n_segments=2, grid_h=4, grid_w=4, has_cls=1,
                            score_mode=0, heads=1, head_dim=8, feat_dim=8, win_rows=2, win_cols=2,
                            keep_global=2, keep_local=4)
    # segment 0: clear scores; segment 1: tokens 1 and 7 (windows 0 and 1) nearly tie for the
    # last global place
    s0 = np.array([16, 3, 15, 2, 1, 4, 0.5, 0.6, 14, 0.7, 13, 0.8, 0.9, 1.1, 1.2, 1.3]) / 100
    s1 = s0.copy()
    s1[7] = s1[1] * (1 - 0.5 * pu.SCORE_RTOL)
    s = np.stack([s0, s1])[None]                       # [1, 2, 16]
    kept = vo.select(s, s, 4, 4, 2, 2, 4, 2)
    ref = {"kept": kept, "scores": s.reshape(1, 32), "scores_local": s.reshape(1, 32)}
    return shape, ref


def test_encoder_kept_rule_on_windows_and_global():
    shape, ref = _enc_case()
    # hand check of the oracle's answer: local = best of each window (0, 2, 8, 10), global = the
    # two best of the rest (5 with 0.04, 1 with 0.03) -> 0 1 2 5 8 10; second segment the same
    assert ref["kept"].tolist() == [[0, 1, 2, 5, 8, 10, 16, 17, 18, 21, 24, 26]]
    assert pu.check_encoder_kept(shape, ref["kept"].copy(), ref, "same") == 0
    # segment 1: token 7 instead of 1 is inside the tolerance -> valid, counted
    alt = ref["kept"].copy()
    alt[0, 6:] = [16, 18, 21, 23, 24, 26]
    assert pu.check_encoder_kept(shape, alt, ref, "near tie") == 1
    # the same swap in segment 0, where the gap is wide -> rejected
    bad = ref["kept"].copy()
    bad[0, :6] = [0, 2, 5, 7, 8, 10]
    with pytest.raises(AssertionError):
        pu.check_encoder_kept(shape, bad, ref, "clear")
    # a window without its local pick (window 1 of segment 1 loses token 18 to token 29) -> rejected
    bad = ref["kept"].copy()
    bad[0, 6:] = [16, 17, 21, 24, 26, 29]
    with pytest.raises(AssertionError):
        pu.check_encoder_kept(shape, bad, ref, "window emptied")
