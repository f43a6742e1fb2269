"""Shared helpers of the parity tests: oracle-side seed screening, host<->device
conversion and the comparison rules.  Nothing here is used by the product path.

Comparison rules (tolerances are stated here once and used by every test):
  * kept indices: bit-exact.
  * scores: relative error of the fp32 GPU scores against the fp64 oracle must
    stay below SCORE_RTOL on every token whose score is not in the deep tail.
  * selection boundaries: a seed is only used when every top-k boundary of the
    oracle (k-th vs (k+1)-th candidate) has a relative gap above MARGIN, which
    is 8x SCORE_RTOL; exact-tie behaviour is tested separately on constructed
    duplicates, where both sides tie exactly.
  * assignment: equal to the oracle's, or the oracle's cosine gap between its
    choice and the GPU's choice is below COS_DELTA (fp32 accumulation cannot
    resolve closer pairs); the number of such tokens is reported.
  * merged features: Eq. 4 evaluated by the oracle under the (validated) GPU
    assignment, rtol 1e-3 (fp32) / 2e-2 (bf16).
  * compacted K / V / hidden: bit-exact (pure copies).
"""
from __future__ import annotations

import numpy as np

from oracle import vscan_oracle as vo
from paper_2505_22654_amd import workloads as wl

SCORE_RTOL = 2e-5
MARGIN = 8 * SCORE_RTOL
COS_DELTA = 1e-5
MERGE_TOL = {wl.F32: dict(rtol=1e-3, atol=1e-6), wl.BF16: dict(rtol=2e-2, atol=1e-5)}


def to_device(a: np.ndarray, dtype: str):
    import torch
    if dtype == wl.BF16:
        return torch.from_numpy(wl.bf16_bits(a)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host(t) -> np.ndarray:
    import torch
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()


def _gap(sorted_desc: np.ndarray, k: int) -> float:
    """Relative gap between the k-th and (k+1)-th best; inf when no boundary exists."""
    if k <= 0 or k >= len(sorted_desc):
        return np.inf
    a, b = sorted_desc[k - 1], sorted_desc[k]
    return (a - b) / a if a > 0 else 0.0


def encoder_boundary_gap(shape, s_local: np.ndarray, s_global: np.ndarray) -> float:
    """Smallest relative gap over all window and global boundaries (oracle scores [B,C,N])."""
    gh, gw, wr, wc = shape.grid_h, shape.grid_w, shape.win_rows, shape.win_cols
    W = wr * wc
    kw = shape.keep_local // W
    kg = shape.keep_global + shape.keep_local - kw * W
    rows = (np.arange(gh) * wr) // gh
    cols = (np.arange(gw) * wc) // gw
    win = (rows[:, None] * wc + cols[None, :]).reshape(-1)
    worst = np.inf
    B, C, N = s_global.shape
    for b in range(B):
        for c in range(C):
            taken = np.zeros(N, bool)
            for w in range(W):
                idx = np.nonzero(win == w)[0]
                order = idx[np.lexsort((idx, -s_local[b, c, idx]))]
                worst = min(worst, _gap(s_local[b, c, order], kw))
                taken[order[:kw]] = True
            rest = np.sort(s_global[b, c, ~taken])[::-1]
            worst = min(worst, _gap(rest, kg))
    return worst


def topk_boundary_gap(scores: np.ndarray, keep: int) -> float:
    worst = np.inf
    for row in scores:
        worst = min(worst, _gap(np.sort(row)[::-1], keep))
    return worst


def screened_encoder_case(shape, seed, logit_gain=1.0, with_local=False, max_tries=16):
    """Inputs + oracle result for the first seed >= `seed` whose boundaries clear MARGIN."""
    for attempt in range(max_tries):
        inp = wl.encoder_inputs(shape, seed + attempt, logit_gain)
        loc = wl.encoder_inputs(shape, seed + attempt, logit_gain, stream=1) if with_local else None
        ref = vo.encoder_reduce(shape, inp["q"], inp["k"], inp["x"],
                                None if loc is None else loc["q"],
                                None if loc is None else loc["k"])
        N = shape.n_tokens
        sg = ref["scores"].reshape(shape.batch, shape.n_segments, N)
        sl = ref["scores_local"].reshape(shape.batch, shape.n_segments, N)
        gap = encoder_boundary_gap(shape, sl, sg)
        if gap > MARGIN:
            return inp, loc, ref, {"seed": seed + attempt, "attempts": attempt + 1, "gap": gap}
    raise AssertionError(f"no seed in {max_tries} tries clears the boundary margin")


def screened_encoder_batch(shape, seed, logit_gain=1.0, max_items=None):
    """Like screened_encoder_case, but screens image by image: the batch is assembled from the
    first `shape.batch` images of the seed's item streams whose boundaries clear MARGIN.  For
    batches with so many boundaries that no whole-batch seed would pass."""
    from dataclasses import replace
    one = replace(shape, batch=1)
    proj = wl.encoder_projections(shape, seed)
    items, refs, tried = [], [], 0
    max_items = max_items or 8 * shape.batch
    N = shape.n_tokens
    while len(items) < shape.batch:
        assert tried < max_items, "too few images clear the boundary margin"
        it = wl.encoder_item(shape, seed, tried, logit_gain, proj)
        tried += 1
        it = {key: it[key][None] for key in ("q", "k", "x")}
        ref = vo.encoder_reduce(one, it["q"], it["k"], it["x"])
        sg = ref["scores"].reshape(1, shape.n_segments, N)
        if encoder_boundary_gap(one, sg, sg) > MARGIN:
            items.append(it)
            refs.append(ref)
    inp = {key: np.concatenate([it[key] for it in items]) for key in ("q", "k", "x")}
    ref = {key: np.concatenate([r[key] for r in refs]) for key in refs[0]}
    return inp, None, ref, {"seed": seed, "images_tried": tried}


def screened_llm_case(shape, seed, max_tries=16):
    for attempt in range(max_tries):
        inp = wl.llm_inputs(shape, seed + attempt)
        ref = vo.llm_prune(shape, **inp)
        gap = topk_boundary_gap(ref["scores"], shape.keep)
        if gap > MARGIN:
            return inp, ref, {"seed": seed + attempt, "attempts": attempt + 1, "gap": gap}
    raise AssertionError(f"no seed in {max_tries} tries clears the boundary margin")


def check_scores(got: np.ndarray, want: np.ndarray, what: str):
    """fp32 scores against fp64 oracle scores, relative, ignoring the deep tail."""
    want = want.reshape(got.shape)
    floor = want.max(axis=-1, keepdims=True) * 1e-30
    mask = want > floor
    rel = np.abs(got.astype(np.float64) - want)[mask] / want[mask]
    worst = rel.max() if rel.size else 0.0
    assert worst < SCORE_RTOL, f"{what}: score relative error {worst:.3e} >= {SCORE_RTOL}"
    return worst


def check_assignment(x: np.ndarray, kept: np.ndarray, got: np.ndarray, want: np.ndarray) -> int:
    """Ambiguity-aware comparison of assignments; returns the number of ambiguous tokens."""
    B, T, D = x.shape
    diff_b, diff_t = np.nonzero(got != want)
    if diff_b.size == 0:
        return 0
    assert got.min() >= 0 and got.max() < kept.shape[1]
    u = diff_b * T + diff_t
    s_want = diff_b * T + kept[diff_b, want[diff_b, diff_t]]
    s_got = diff_b * T + kept[diff_b, got[diff_b, diff_t]]
    flat = x.reshape(B * T, D)
    gap = vo.cos_pairs(flat, u, s_want) - vo.cos_pairs(flat, u, s_got)
    assert np.all(gap >= 0) and gap.max() < COS_DELTA, (
        f"{diff_b.size} assignments differ, worst oracle cosine gap {gap.max():.3e}")
    return int(diff_b.size)


def check_encoder(shape, inp, ref, out, what=""):
    """Full comparison of one vscan_encoder_reduce result with the oracle."""
    kept = to_host(out["kept_idx"])
    assert np.array_equal(kept, ref["kept"]), f"{what}: kept indices differ"
    report = {}
    if "scores" in out:
        report["score_rel_err"] = check_scores(to_host(out["scores"]), ref["scores"], what)
    assign = to_host(out["assign"])
    report["ambiguous"] = check_assignment(inp["x"], kept, assign, ref["assign"])
    merged_ref, _ = vo.merge(inp["x"], kept, assign)
    np.testing.assert_allclose(to_host(out["merged"]).astype(np.float64), merged_ref,
                               err_msg=f"{what}: merged", **MERGE_TOL[shape.dtype])
    return report


def check_llm(shape, inp, ref, out, what=""):
    kept = to_host(out["kept_idx"])
    assert np.array_equal(kept, ref["kept"]), f"{what}: kept indices differ"
    report = {}
    if "scores" in out:
        report["score_rel_err"] = check_scores(to_host(out["scores"]), ref["scores"], what)
    for name in ("k", "v", "hidden"):
        got = to_host(out[name])
        assert got.shape == ref[name].shape, f"{what}: {name} shape"
        assert np.array_equal(got, ref[name]), f"{what}: compacted {name} differs"
    return report


def ragged_llm_case(base, seqs, seed):
    """A ragged stage-2 batch.  `base`: an LlmShape giving the shared fields; `seqs`: list of
    (prefix, vis_len, text, keep).  Every sequence is generated and screened on its own (batch-1
    shapes) and padded with noise to the common capacity.  Returns the capacity shape, the meta
    rows (seq_len, vis_start, vis_len, keep), the padded inputs and the per-sequence oracle
    results."""
    from dataclasses import replace
    cap_S = max(p + v + t for p, v, t, _ in seqs)
    cap_V = max(v for _, v, _, _ in seqs)
    cap_keep = max(kp for *_, kp in seqs)
    caps = replace(base, batch=len(seqs), prefix=0, vis_len=cap_V, text=cap_S - cap_V,
                   keep=cap_keep)
    rng = np.random.default_rng(seed)
    H, Hq, dh, Dh, Tq = base.kv_heads, base.q_heads, base.head_dim, base.hidden, base.n_query
    pad = lambda *shape: wl._finish(rng.standard_normal(shape).astype(np.float32), base.dtype)
    inp = {"q": np.empty((len(seqs), Hq, Tq, dh), np.float32), "k": pad(len(seqs), H, cap_S, dh),
           "v": pad(len(seqs), H, cap_S, dh), "hidden": pad(len(seqs), cap_S, Dh)}
    meta, refs = [], []
    for b, (p, v, t, kp) in enumerate(seqs):
        one = replace(base, batch=1, prefix=p, vis_len=v, text=t, keep=kp)
        for attempt in range(32):
            item = wl.llm_inputs(one, seed + 100 * b + attempt)
            ref = vo.llm_prune(one, **item)
            if topk_boundary_gap(ref["scores"], kp) > MARGIN:
                break
        else:
            raise AssertionError("no seed clears the boundary margin")
        S = one.seq_len
        inp["q"][b] = item["q"][0]
        inp["k"][b, :, :S] = item["k"][0]
        inp["v"][b, :, :S] = item["v"][0]
        inp["hidden"][b, :S] = item["hidden"][0]
        meta.append((S, p, v, kp))
        refs.append(ref)
    return caps, meta, inp, refs


def check_llm_ragged(caps, meta, inp, refs, out, in_place, what=""):
    """Per sequence against the oracle; entries and rows outside a sequence's result must be
    the padding value (-1 for indices) or untouched."""
    kept = to_host(out["kept_idx"])
    scores = to_host(out["scores"]) if "scores" in out else None
    got = {n: to_host(out[n]) for n in ("k", "v", "hidden")}
    worst = 0.0
    for b, (S, vs, V, kp) in enumerate(meta):
        ref = refs[b]
        assert np.array_equal(kept[b, :kp], ref["kept"][0]), f"{what}[{b}]: kept indices differ"
        assert np.all(kept[b, kp:] == -1), f"{what}[{b}]: index padding"
        if scores is not None:
            worst = max(worst, check_scores(scores[b:b + 1, :V], ref["scores"], f"{what}[{b}]"))
        So = S - V + kp
        assert np.array_equal(got["k"][b, :, :So], ref["k"][0]), f"{what}[{b}]: k"
        assert np.array_equal(got["v"][b, :, :So], ref["v"][0]), f"{what}[{b}]: v"
        assert np.array_equal(got["hidden"][b, :So], ref["hidden"][0]), f"{what}[{b}]: hidden"
        if in_place:  # rows past the sequence's own length are never touched
            assert np.array_equal(got["k"][b, :, S:], inp["k"][b, :, S:]), f"{what}[{b}]: k padding"
            assert np.array_equal(got["hidden"][b, S:], inp["hidden"][b, S:]), f"{what}[{b}]: hidden padding"
        else:         # the binding zero-fills the destinations; rows past the result stay zero
            assert not got["k"][b, :, So:].any() and not got["hidden"][b, So:].any(), \
                f"{what}[{b}]: rows past the result were written"
    return {"score_rel_err": worst}


def fused_reference(shape, hidden, w_q, w_k):
    return vo.llm_prune_fused(shape, hidden, w_q, w_k)


def screened_fused_case(shape, seed, max_tries=16):
    """Hidden states and projection weights whose oracle selection clears the margin."""
    for attempt in range(max_tries):
        hidden = wl.llm_inputs(shape, seed + attempt)["hidden"]
        w = wl.llm_weights(shape, seed + attempt)
        ref = fused_reference(shape, hidden, w["w_q"], w["w_k"])
        gap = topk_boundary_gap(ref["scores"], shape.keep)
        if gap > MARGIN:
            inp = {"hidden": hidden, "w_q": w["w_q"], "w_k": w["w_k"]}
            return inp, ref, {"seed": seed + attempt, "attempts": attempt + 1, "gap": gap}
    raise AssertionError(f"no seed in {max_tries} tries clears the boundary margin")


def check_fused(shape, ref, out, what=""):
    kept = to_host(out["kept_idx"])
    assert np.array_equal(kept, ref["kept"]), f"{what}: kept indices differ"
    report = {}
    if "scores" in out:
        report["score_rel_err"] = check_scores(to_host(out["scores"]), ref["scores"], what)
    got = to_host(out["hidden"])
    assert got.shape == ref["hidden"].shape, f"{what}: hidden shape"
    assert np.array_equal(got, ref["hidden"]), f"{what}: compacted hidden differs"
    return report


def screened_encoder_fused_case(shape, seed, logit_gain=1.0, with_local=False, max_tries=16):
    """Hidden rows, weights and oracle result for the first seed whose boundaries clear MARGIN."""
    for attempt in range(max_tries):
        inp = wl.encoder_hidden_inputs(shape, seed + attempt, logit_gain)
        loc = (wl.encoder_hidden_inputs(shape, seed + attempt, logit_gain, stream=1)
               if with_local else None)
        ref = vo.encoder_reduce_fused(shape, inp["hidden"], inp["w_q"], inp["w_k"], inp["x"],
                                      *((loc["hidden"], loc["w_q"], loc["w_k"]) if loc else ()))
        N = shape.n_tokens
        sg = ref["scores"].reshape(shape.batch, shape.n_segments, N)
        sl = ref["scores_local"].reshape(shape.batch, shape.n_segments, N)
        gap = encoder_boundary_gap(shape, sl, sg)
        if gap > MARGIN:
            return inp, loc, ref, {"seed": seed + attempt, "attempts": attempt + 1, "gap": gap}
    raise AssertionError(f"no seed in {max_tries} tries clears the boundary margin")


def ragged_fused_case(base, seqs, seed):
    """A ragged batch for the stage-2 form that scores from hidden states.  `seqs`: list of
    (prefix, vis_len, text, keep).  One set of weights; every sequence is generated and screened
    on its own (batch-1 shapes) and padded with noise to the common capacity."""
    from dataclasses import replace
    cap_S = max(p + v + t for p, v, t, _ in seqs)
    cap_V = max(v for _, v, _, _ in seqs)
    caps = replace(base, batch=len(seqs), prefix=0, vis_len=cap_V, text=cap_S - cap_V,
                   keep=max(kp for *_, kp in seqs))
    rng = np.random.default_rng(seed)
    w = wl.llm_weights(base, seed)
    hidden = wl._finish(rng.standard_normal((len(seqs), cap_S, base.hidden)).astype(np.float32),
                        base.dtype)
    meta, refs = [], []
    for b, (p, v, t, kp) in enumerate(seqs):
        one = replace(base, batch=1, prefix=p, vis_len=v, text=t, keep=kp)
        for attempt in range(32):
            item = wl.llm_inputs(one, seed + 100 * b + attempt)["hidden"]
            ref = vo.llm_prune_fused(one, item, w["w_q"], w["w_k"])
            if topk_boundary_gap(ref["scores"], kp) > MARGIN:
                break
        else:
            raise AssertionError("no seed clears the boundary margin")
        hidden[b, :one.seq_len] = item[0]
        meta.append((one.seq_len, p, v, kp))
        refs.append(ref)
    return caps, meta, {"hidden": hidden, "w_q": w["w_q"], "w_k": w["w_k"]}, refs


def check_fused_ragged(caps, meta, inp, refs, out, in_place, what=""):
    kept = to_host(out["kept_idx"])
    scores = to_host(out["scores"])
    got = to_host(out["hidden"])
    worst = 0.0
    for b, (S, vs, V, kp) in enumerate(meta):
        ref = refs[b]
        assert np.array_equal(kept[b, :kp], ref["kept"][0]), f"{what}[{b}]: kept indices differ"
        assert np.all(kept[b, kp:] == -1), f"{what}[{b}]: index padding"
        worst = max(worst, check_scores(scores[b:b + 1, :V], ref["scores"], f"{what}[{b}]"))
        So = S - V + kp
        assert np.array_equal(got[b, :So], ref["hidden"][0]), f"{what}[{b}]: hidden"
        if in_place:
            assert np.array_equal(got[b, S:], inp["hidden"][b, S:]), f"{what}[{b}]: padding rows"
        else:
            assert not got[b, So:].any(), f"{what}[{b}]: rows past the result were written"
    return {"score_rel_err": worst}
