"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Rules and tolerances live in tests/parity_utils.py."""
import dataclasses

import numpy as np
import pytest

from oracle import vscan_oracle as vo
from paper_2505_22654_amd import binding as vb
from paper_2505_22654_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu


def _run_encoder(shape, inp, loc=None):
    q, k, x = (pu.to_device(inp[n], shape.dtype) for n in ("q", "k", "x"))
    ql = kl = None
    if loc is not None:
        ql, kl = pu.to_device(loc["q"], shape.dtype), pu.to_device(loc["k"], shape.dtype)
    import torch
    out = vb.encoder_reduce(shape, q, k, x, ql, kl, want_assign=True, want_scores=True)
    torch.cuda.synchronize()
    return out


def _run_llm(shape, inp):
    import torch
    q, k, v, h = (pu.to_device(inp[n], shape.dtype) for n in ("q", "k", "v", "hidden"))
    out = vb.llm_prune(shape, q, k, v, h, want_scores=True)
    torch.cuda.synchronize()
    return out


def _enc(dtype=wl.BF16, **kw):
    base = dict(dtype=dtype, batch=2, n_segments=1, grid_h=12, grid_w=12, has_cls=1, score_mode=0,
                heads=4, head_dim=32, feat_dim=128, win_rows=2, win_cols=2, keep_global=10,
                keep_local=8)
    base.update(kw)
    return wl.EncoderShape(**base)


SMALL_ENCODER = {
    # several tiles and a ragged tail in every dimension
    "bf16-ragged": _enc(batch=3, n_segments=2, grid_h=13, grid_w=11, heads=3, head_dim=40,
                        feat_dim=200, win_rows=3, win_cols=2, keep_global=17, keep_local=13),
    "f32-ragged": _enc(wl.F32, batch=2, n_segments=3, grid_h=9, grid_w=14, heads=5, head_dim=24,
                       feat_dim=136, win_rows=2, win_cols=3, keep_global=9, keep_local=12),
    "bf16-all-keys": _enc(softmax_domain=1, keep_global=30, keep_local=16),
    "f32-all-keys": _enc(wl.F32, softmax_domain=1),
    "bf16-one-window": _enc(win_rows=1, win_cols=1, keep_local=5, keep_global=0),
    "bf16-global-only": _enc(keep_local=0, keep_global=21),
    "bf16-many-kept": _enc(grid_h=20, grid_w=20, keep_global=150, keep_local=100, feat_dim=264),
    "bf16-wide-rows": _enc(head_dim=256, feat_dim=1032, heads=2),
    # feature rows near the 16 KiB limit: every lane of the merge owns up to 16 pieces
    "bf16-widest-rows": _enc(feat_dim=8192, heads=2, grid_h=10, grid_w=9, keep_global=7,
                             keep_local=8),
    "f32-widest-rows": _enc(wl.F32, feat_dim=4088, heads=2, grid_h=9, grid_w=10, keep_global=6,
                            keep_local=4),
    "f32-keep-one": _enc(wl.F32, keep_global=1, keep_local=0),
    "bf16-mean": _enc(has_cls=0, score_mode=1, grid_h=15, grid_w=13, head_dim=80, heads=3,
                      win_rows=3, win_cols=3, keep_global=20, keep_local=18),
    "bf16-mean-cls-all-keys": _enc(has_cls=1, score_mode=1, softmax_domain=1, grid_h=16,
                                   grid_w=20, head_dim=64),
    "bf16-mean-cls": _enc(has_cls=1, score_mode=1, grid_h=11, grid_w=12, head_dim=48),
    "f32-mean": _enc(wl.F32, has_cls=0, score_mode=1, grid_h=14, grid_w=10, head_dim=40),
    "bf16-mean-wide": _enc(has_cls=0, score_mode=1, grid_h=18, grid_w=9, head_dim=160, heads=2),
    # more than 1024 tokens per segment: the workgroup-wide threshold search
    "bf16-large-grid": _enc(grid_h=40, grid_w=37, heads=2, feat_dim=64, win_rows=5, win_cols=4,
                            keep_global=130, keep_local=100),
    "f32-large-grid-one-window": _enc(wl.F32, batch=1, grid_h=33, grid_w=35, heads=2, feat_dim=64,
                                      win_rows=1, win_cols=1, keep_global=7, keep_local=300),
    "bf16-odd-head-dim-cls": _enc(head_dim=80, heads=3, keep_global=12, keep_local=12),
}


@pytest.mark.parametrize("name", sorted(SMALL_ENCODER))
def test_encoder_small(name):
    shape = SMALL_ENCODER[name]
    # peakier scores on the big grids: thousands of candidates leave few seeds with a clear
    # boundary when the scores are flat
    gain = 1.0 if "large" in name else 0.25
    inp, _, ref, info = pu.screened_encoder_case(shape, seed=1000 + len(name), logit_gain=gain)
    out = _run_encoder(shape, inp)
    rep = pu.check_encoder(shape, inp, ref, out, name)
    print(name, info, rep)


def test_encoder_local_scan_from_shallow_layer_pair():
    shape = _enc(batch=2, n_segments=2, grid_h=12, grid_w=12, keep_global=12, keep_local=12)
    inp, loc, ref, info = pu.screened_encoder_case(shape, seed=77, logit_gain=0.25, with_local=True)
    assert not np.array_equal(ref["scores"], ref["scores_local"])
    out = _run_encoder(shape, inp, loc)
    pu.check_encoder(shape, inp, ref, out, "local-pair")


def test_encoder_local_pair_on_a_large_segment():
    """More than 4096 tokens per segment: the local scan runs window by window in a kernel of its
    own, here on the scores of the shallow-layer pair, and hands keys and flags to the global scan."""
    shape = _enc(batch=1, n_segments=2, grid_h=80, grid_w=80, heads=2, head_dim=16, feat_dim=32,
                 win_rows=4, win_cols=4, keep_global=40, keep_local=48)
    inp, loc, ref, info = pu.screened_encoder_case(shape, seed=78, logit_gain=1.0, with_local=True,
                                                   max_tries=4)
    out = _run_encoder(shape, inp, loc)
    print("local-pair-large", info, pu.check_encoder(shape, inp, ref, out, "local-pair-large"))


@pytest.mark.parametrize("dtype,feat_dim", [(wl.BF16, 1032), (wl.BF16, 2048), (wl.F32, 520)])
def test_encoder_clustered_features_make_very_large_groups(dtype, feat_dim):
    """Features drawn around five prototypes: dozens of groups of 33-128 members (shared by the
    waves of a workgroup) and at least one of more than 128 (longer than a slot's list, gathered
    by a scan of the token range), on rows wide enough to be added as two column halves."""
    shape = _enc(dtype, batch=2, n_segments=1, grid_h=40, grid_w=37, heads=2, head_dim=32,
                 feat_dim=feat_dim, win_rows=2, win_cols=2, keep_global=30, keep_local=20)
    inp = wl.encoder_inputs(shape, 77)
    rng = np.random.default_rng(5)
    T = shape.grid_h * shape.grid_w
    protos = rng.standard_normal((5, feat_dim)).astype(np.float32)
    which = rng.integers(0, 5, size=(shape.batch, T))
    x = protos[which] + 0.05 * rng.standard_normal((shape.batch, T, feat_dim)).astype(np.float32)
    inp["x"] = wl.round_to_bf16(x) if dtype == wl.BF16 else x
    ref = vo.encoder_reduce(shape, inp["q"], inp["k"], inp["x"])
    sizes = np.concatenate([np.bincount(ref["assign"][b], minlength=shape.keep)
                            for b in range(shape.batch)])
    assert sizes.max() > 128 and (sizes > 32).sum() >= 10, sizes.max()
    out = _run_encoder(shape, inp)
    print("clustered", pu.check_encoder(shape, inp, ref, out, "clustered"))
    again = _run_encoder(shape, inp)  # shared groups and column halves add in a fixed order
    for name in ("kept_idx", "merged", "assign"):
        assert np.array_equal(pu.to_host(out[name]), pu.to_host(again[name])), name


def test_encoder_long_image_merge_by_sixteen_waves_and_column_halves():
    """9216 tokens, 2048 kept: the merge runs with sixteen-wave workgroups, and with 128 of them
    per column half both halves fit one round (config 4 has too many for that); clustered
    features give it groups of more than 128 members."""
    shape = _enc(wl.BF16, batch=1, n_segments=1, grid_h=96, grid_w=96, heads=2, head_dim=16,
                 feat_dim=1024, win_rows=4, win_cols=4, keep_global=1024, keep_local=1024)
    inp = wl.encoder_inputs(shape, 78)
    rng = np.random.default_rng(6)
    T = shape.grid_h * shape.grid_w
    protos = rng.standard_normal((5, shape.feat_dim)).astype(np.float32)
    which = rng.integers(0, 5, size=(shape.batch, T))
    x = protos[which] + 0.05 * rng.standard_normal((shape.batch, T, shape.feat_dim)).astype(np.float32)
    inp["x"] = wl.round_to_bf16(x)
    ref = vo.encoder_reduce(shape, inp["q"], inp["k"], inp["x"])
    sizes = np.bincount(ref["assign"][0], minlength=shape.keep)
    assert sizes.max() > 128, sizes.max()
    out = _run_encoder(shape, inp)
    print("long-image", sizes.max(), pu.check_encoder(shape, inp, ref, out, "long-image"))
    again = _run_encoder(shape, inp)
    for name in ("kept_idx", "merged", "assign"):
        assert np.array_equal(pu.to_host(out[name]), pu.to_host(again[name])), name


def test_encoder_keep_everything_is_identity():
    shape = _enc(wl.F32, grid_h=8, grid_w=8, keep_global=32, keep_local=32)
    inp = wl.encoder_inputs(shape, 5)
    out = _run_encoder(shape, inp)
    assert np.array_equal(pu.to_host(out["kept_idx"]), np.arange(64)[None].repeat(2, 0))
    assert np.array_equal(pu.to_host(out["merged"]), inp["x"])
    assert np.array_equal(pu.to_host(out["assign"]), np.arange(64)[None].repeat(2, 0))


def test_encoder_exact_ties():
    """q = 0 gives every token the same score on both sides: the result must be the first
    kw row-major tokens of every window, then the lowest remaining indices; duplicated
    kept rows must send their copies to the lowest slot."""
    shape = _enc(wl.F32, batch=1, grid_h=8, grid_w=8, win_rows=2, win_cols=2, keep_global=3,
                 keep_local=8, feat_dim=64)
    inp = wl.encoder_inputs(shape, 9)
    inp["q"][:] = 0.0
    x = inp["x"]
    x[0, 2] = x[0, 0]        # tokens 0 and 2 are kept (see below) and identical
    x[0, 40] = x[0, 0]       # a dropped copy -> must go to slot 0, not slot 2
    ref = vo.encoder_reduce(shape, inp["q"], inp["k"], x)
    want = sorted([0, 1, 4, 5, 32, 33, 36, 37] + [2, 3, 6])
    assert ref["kept"].tolist() == [want]
    out = _run_encoder(shape, inp)
    assert pu.to_host(out["kept_idx"]).tolist() == [want]
    assign = pu.to_host(out["assign"])
    assert assign[0, 40] == 0 and ref["assign"][0, 40] == 0
    pu.check_encoder(shape, inp, ref, out, "ties")


def test_encoder_exact_ties_large_grid():
    """All scores tie on a segment large enough for the workgroup-wide threshold search."""
    shape = _enc(wl.F32, batch=1, grid_h=36, grid_w=40, win_rows=3, win_cols=4, keep_global=101,
                 keep_local=50, feat_dim=32, heads=2)
    inp = wl.encoder_inputs(shape, 11)
    inp["q"][:] = 0.0
    ref = vo.encoder_reduce(shape, inp["q"], inp["k"], inp["x"])
    out = _run_encoder(shape, inp)
    assert np.array_equal(pu.to_host(out["kept_idx"]), ref["kept"])
    pu.check_encoder(shape, inp, ref, out, "ties-large")


@pytest.mark.parametrize("win,keep_local,keep_global", [(4, 50, 301), (1, 0, 777)])
def test_encoder_exact_ties_on_a_segment_split_over_workgroups(win, keep_local, keep_global):
    """All scores tie on a segment of more than 4096 tokens: the local scan of every window
    (a kernel of its own there) and the workgroup-wide global search must both fall back on the
    token order; with one window the segment is cut into runs of 1024 tokens instead."""
    shape = _enc(wl.F32, batch=1, n_segments=2, grid_h=72, grid_w=64, win_rows=win, win_cols=win,
                 keep_global=keep_global, keep_local=keep_local, feat_dim=32, heads=2, head_dim=16)
    inp = wl.encoder_inputs(shape, 12)
    inp["q"][:] = 0.0
    ref = vo.encoder_reduce(shape, inp["q"], inp["k"], inp["x"])
    out = _run_encoder(shape, inp)
    assert np.array_equal(pu.to_host(out["kept_idx"]), ref["kept"])
    pu.check_encoder(shape, inp, ref, out, "ties-split")


def test_encoder_runs_are_bit_reproducible():
    shape = SMALL_ENCODER["bf16-ragged"]
    inp = wl.encoder_inputs(shape, 3, 0.25)
    a, b = _run_encoder(shape, inp), _run_encoder(shape, inp)
    for name in ("kept_idx", "merged", "assign", "scores"):
        assert np.array_equal(pu.to_host(a[name]), pu.to_host(b[name])), name


def _llm(dtype=wl.BF16, **kw):
    base = dict(dtype=dtype, batch=2, prefix=5, vis_len=50, text=9, n_query=1, q_heads=4,
                kv_heads=4, head_dim=32, hidden=64, keep=20)
    base.update(kw)
    return wl.LlmShape(**base)


SMALL_LLM = {
    "bf16-basic": _llm(),
    "f32-basic": _llm(wl.F32),
    "bf16-gqa-queries": _llm(batch=3, q_heads=12, kv_heads=4, n_query=3, vis_len=333, text=17,
                             head_dim=40, hidden=200, keep=111),
    "f32-gqa": _llm(wl.F32, q_heads=6, kv_heads=2, vis_len=77, head_dim=24, hidden=136, keep=30),
    "bf16-many-rows": _llm(q_heads=8, kv_heads=2, n_query=8, vis_len=130, text=20, keep=64),
    "bf16-causal-domain": _llm(softmax_domain=1, n_query=4, q_heads=8, kv_heads=4, text=12),
    "f32-causal-domain": _llm(wl.F32, softmax_domain=1, n_query=2, text=6),
    "bf16-in-place": _llm(in_place=1, batch=3, vis_len=300, text=40, keep=100, head_dim=128,
                          hidden=520),
    "f32-in-place": _llm(wl.F32, in_place=1, vis_len=200, text=33, keep=7, head_dim=64,
                         hidden=264),
    "bf16-keep-all": _llm(keep=50),
    "bf16-keep-all-in-place": _llm(keep=50, in_place=1),
    "bf16-keep-none": _llm(keep=0),
    "bf16-no-prefix": _llm(prefix=0, in_place=1),
    # more than 1024 visual tokens: the workgroup-wide threshold search
    "bf16-large-span": _llm(vis_len=1500, text=30, keep=700, in_place=1, hidden=128),
    "f32-large-span": _llm(wl.F32, vis_len=1111, text=5, keep=3, hidden=72),
}


@pytest.mark.parametrize("name", sorted(SMALL_LLM))
def test_llm_small(name):
    shape = SMALL_LLM[name]
    inp, ref, info = pu.screened_llm_case(shape, seed=2000 + len(name))
    out = _run_llm(shape, inp)
    rep = pu.check_llm(shape, inp, ref, out, name)
    print(name, info, rep)


def test_llm_max_span():
    """A visual span close to the largest the stage-2 select takes (keys and flags of one
    sequence fill LDS), in place; the next size up is refused."""
    shape = _llm(batch=2, prefix=3, vis_len=32500, text=5, q_heads=1, kv_heads=1, head_dim=16,
                 hidden=16, keep=150, n_query=1, in_place=1)
    inp, ref, info = pu.screened_llm_case(shape, seed=9100)
    print("max-span", info, pu.check_llm(shape, inp, ref, _run_llm(shape, inp), "max-span"))
    with pytest.raises(vb.VscanError) as e:
        vb.llm_workspace_size(vb.llm_desc(dataclasses.replace(shape, vis_len=32700)))
    assert e.value.status == vb.VSCAN_ERR_UNSUPPORTED


def test_llm_multi_turn_reselection():
    """A second question re-scores the same unpruned pool (App. "Remarks on Multi-Turn
    Conversations"): out-of-place pruning leaves hidden states and K/V untouched, and each turn's result
    matches the oracle for that turn's queries."""
    import torch
    shape = _llm(batch=3, prefix=5, vis_len=333, text=40, keep=77, n_query=2)
    inp1, ref1, info1 = pu.screened_llm_case(shape, seed=4100)
    inp2, ref2, info2 = pu.screened_llm_case(shape, seed=4200)
    # turn 2 = turn 1's pool with turn 2's queries
    turn2 = dict(inp1, q=inp2["q"])
    ref_t2 = vo.llm_prune(shape, **turn2)  # a close boundary falls to check_llm's validity check
    q1, k, v, h = (pu.to_device(inp1[n], shape.dtype) for n in ("q", "k", "v", "hidden"))
    q2 = pu.to_device(inp2["q"], shape.dtype)
    pool = [t.clone() for t in (k, v, h)]
    out1 = vb.llm_prune(shape, q1, k, v, h, want_scores=True)
    out2 = vb.llm_prune(shape, q2, k, v, h, want_scores=True)
    torch.cuda.synchronize()
    for before, after in zip(pool, (k, v, h)):
        assert torch.equal(before, after), "out-of-place pruning modified the pool"
    print("turn 1", info1, pu.check_llm(shape, inp1, ref1, out1, "turn1"))
    print("turn 2", pu.check_llm(shape, turn2, ref_t2, out2, "turn2"))
    assert not np.array_equal(pu.to_host(out1["kept_idx"]), pu.to_host(out2["kept_idx"]))


RAGGED_SEQS = [
    # (prefix, vis_len, text, keep): long and short spans, nothing kept, everything kept,
    # a span shorter than one tile, the longest sequence not the one with the longest span
    (35, 900, 70, 300), (3, 5, 9, 2), (0, 333, 41, 0), (12, 257, 300, 257), (7, 1100, 13, 1),
    (20, 64, 20, 63),
]


@pytest.mark.parametrize("variant", ["bf16", "bf16-inplace", "f32-all-keys", "bf16-gqa-inplace"])
def test_llm_ragged(variant):
    """Per-sequence lengths, spans and budgets in one call (dynamic-resolution inputs,
    Sec. 5.1 "Models"), each sequence against the oracle run on that sequence alone."""
    import torch
    base = {
        "bf16": _llm(n_query=1),
        "bf16-inplace": _llm(in_place=1, n_query=2),
        "f32-all-keys": _llm(wl.F32, softmax_domain=1, head_dim=64, n_query=1),
        "bf16-gqa-inplace": _llm(in_place=1, q_heads=8, kv_heads=2, head_dim=128, n_query=3),
    }[variant]
    caps, meta, inp, refs = pu.ragged_llm_case(base, RAGGED_SEQS, seed=7000 + len(variant))
    q, k, v, h = (pu.to_device(inp[n], caps.dtype) for n in ("q", "k", "v", "hidden"))
    out = vb.llm_prune_ragged(caps, meta, q, k, v, h, want_scores=True)
    torch.cuda.synchronize()
    print(variant, pu.check_llm_ragged(caps, meta, inp, refs, out, caps.in_place, variant))


def test_llm_ragged_matches_uniform():
    """A ragged call whose sequences all have the descriptor's own lengths gives exactly what
    the uniform entry point gives."""
    import torch
    shape = _llm(batch=4, prefix=9, vis_len=400, text=33, keep=100, n_query=2)
    inp, ref, info = pu.screened_llm_case(shape, seed=7300)
    q, k, v, h = (pu.to_device(inp[n], shape.dtype) for n in ("q", "k", "v", "hidden"))
    uni = vb.llm_prune(shape, q, k, v, h, want_scores=True)
    meta = [(shape.seq_len, shape.vis_start, shape.vis_len, shape.keep)] * shape.batch
    rag = vb.llm_prune_ragged(shape, meta, q, k, v, h, want_scores=True)
    torch.cuda.synchronize()
    So = shape.seq_out
    assert torch.equal(uni["kept_idx"], rag["kept_idx"]) and torch.equal(uni["scores"], rag["scores"])
    assert torch.equal(uni["k"], rag["k"][:, :, :So]) and torch.equal(uni["v"], rag["v"][:, :, :So])
    assert torch.equal(uni["hidden"], rag["hidden"][:, :So])
    print("ragged == uniform", info, pu.check_llm(shape, inp, ref, uni, "uniform"))


@pytest.mark.parametrize("pattern", ["last", "first", "alternate"])
def test_in_place_compaction_hazards(pattern):
    """Steer the selection (by planting large keys) to the patterns that stress the
    write-after-read hazard of in-place compaction, and compare with out-of-place."""
    shape = _llm(in_place=1, batch=2, prefix=3, vis_len=700, text=300, keep=350, head_dim=128,
                 hidden=256, q_heads=2, kv_heads=2)
    inp = wl.llm_inputs(shape, 31)
    V = shape.vis_len
    chosen = {"last": np.arange(V - shape.keep, V), "first": np.arange(shape.keep),
              "alternate": np.arange(0, V, 2)}[pattern]
    qdir = inp["q"].mean(axis=(1, 2))                      # [B, dh]
    for b in range(shape.batch):
        inp["k"][b][:, shape.vis_start + chosen] += wl.round_to_bf16(4.0 * qdir[b])
    inp["k"] = wl.round_to_bf16(inp["k"])
    ref = vo.llm_prune(shape, **inp)
    assert np.array_equal(ref["kept"], chosen[None].repeat(shape.batch, 0))
    out = _run_llm(shape, inp)
    pu.check_llm(shape, inp, ref, out, pattern)
    out2 = _run_llm(dataclasses.replace(shape, in_place=0), inp)
    for name in ("k", "v", "hidden"):
        assert np.array_equal(pu.to_host(out[name]), pu.to_host(out2[name]))


def test_llm_exact_ties_keep_first_tokens():
    shape = _llm(wl.F32, keep=13)
    inp = wl.llm_inputs(shape, 4)
    inp["k"][:] = 1.0
    ref = vo.llm_prune(shape, **inp)
    assert ref["kept"].tolist() == [list(range(13))] * 2
    out = _run_llm(shape, inp)
    pu.check_llm(shape, inp, ref, out, "ties")


def test_llm_exact_ties_large_span():
    shape = _llm(wl.F32, vis_len=1300, keep=401, text=3)
    inp = wl.llm_inputs(shape, 4)
    inp["k"][:] = 1.0
    ref = vo.llm_prune(shape, **inp)
    assert ref["kept"].tolist() == [list(range(401))] * 2
    pu.check_llm(shape, inp, ref, _run_llm(shape, inp), "ties-large")


def _expected_by_groups(group_of, group_score, keep):
    """Tokens whose scores tie exactly inside each group: the best groups whole, then the
    lowest indices of the group the budget ends in."""
    order = np.argsort(-group_score, kind="stable")
    picked = []
    for g in order:
        members = np.flatnonzero(group_of == g)
        take = min(len(members), keep - len(picked))
        picked.extend(members[:take].tolist())
        if len(picked) == keep:
            break
    return sorted(picked)


def _group_scores(scores, group_of, n_groups):
    """Per group score from the oracle; the groups must be far apart next to rounding."""
    gs = np.array([scores[group_of == g].mean() for g in range(n_groups)])
    for g in range(n_groups):
        assert np.ptp(scores[group_of == g]) <= 1e-9 * gs[g]
    srt = np.sort(gs)
    return gs, float(np.min(np.diff(srt) / srt[1:])) if n_groups > 1 else 1.0


@pytest.mark.parametrize("n_groups", [2, 24, 100])
def test_llm_tied_groups_go_to_the_lowest_tokens(n_groups):
    """Visual keys drawn from a few distinct rows: scores tie exactly inside a group, and the
    budget ends inside one, so the workgroup-wide search has to settle a tie that covers only
    part of the candidates (2 groups of about 1500 tokens, 24 of about 125, 100 of about 30)
    by token order."""
    shape = _llm(wl.F32, batch=2, vis_len=3000, keep=1000, text=5)
    inp = wl.llm_inputs(shape, 21)
    rng = np.random.default_rng(100 + n_groups)
    group_of = rng.integers(0, n_groups, size=shape.vis_len)
    for attempt in range(20):
        rows = rng.standard_normal((shape.batch, shape.kv_heads, n_groups, shape.head_dim)).astype(np.float32)
        inp["k"][:, :, shape.vis_start:shape.vis_start + shape.vis_len] = rows[:, :, group_of]
        ref = vo.llm_prune(shape, **inp)
        per_seq = [_group_scores(ref["scores"][b], group_of, n_groups) for b in range(shape.batch)]
        if min(gap for _, gap in per_seq) > 3e-5:  # fp32 scores are good to about 1e-6
            break
    else:
        pytest.fail("no draw with well separated groups")
    want = [_expected_by_groups(group_of, gs, shape.keep) for gs, _ in per_seq]
    out = _run_llm(shape, inp)
    assert pu.to_host(out["kept_idx"]).tolist() == want
    pu.check_scores(pu.to_host(out["scores"]), ref["scores"], "tied-groups")


@pytest.mark.parametrize("grid,n_groups", [((40, 40), 12), ((72, 64), 40), ((72, 64), 3)])
def test_encoder_tied_groups_go_to_the_lowest_tokens(grid, n_groups):
    """The same for the encoder's global scan, on a segment searched by one workgroup (1600
    tokens) and on one split over workgroups (4608 tokens); no local scan, so the expected
    selection follows from the groups alone."""
    shape = _enc(wl.F32, batch=1, n_segments=2, grid_h=grid[0], grid_w=grid[1], win_rows=1,
                 win_cols=1, keep_local=0, keep_global=grid[0] * grid[1] // 3, feat_dim=32,
                 heads=2, head_dim=16)
    N = grid[0] * grid[1]
    inp = wl.encoder_inputs(shape, 31)
    rng = np.random.default_rng(200 + n_groups)
    group_of = rng.integers(0, n_groups, size=N)
    for attempt in range(20):
        rows = rng.standard_normal((1, shape.n_segments, shape.heads, n_groups, shape.head_dim)).astype(np.float32)
        inp["k"][:, :, :, shape.has_cls:] = rows[:, :, :, group_of]
        ref = vo.encoder_reduce(shape, inp["q"], inp["k"], inp["x"])
        per_seg = [_group_scores(ref["scores"][0, c * N:(c + 1) * N], group_of, n_groups)
                   for c in range(shape.n_segments)]
        if min(gap for _, gap in per_seg) > 3e-5:
            break
    else:
        pytest.fail("no draw with well separated groups")
    want = []
    for c, (gs, _) in enumerate(per_seg):
        want += [c * N + j for j in _expected_by_groups(group_of, gs, shape.keep_global)]
    out = _run_encoder(shape, inp)
    assert pu.to_host(out["kept_idx"]).tolist() == [want]
    pu.check_scores(pu.to_host(out["scores"]), ref["scores"], "tied-groups")


# ----------------------------------------------------------------------------
# The benchmark configurations at full size
@pytest.mark.parametrize("win,keep_local,keep_global", [(2, 12, 20), (1, 0, 32), (6, 36, 20)])
def test_encoder_max_segment(win, keep_local, keep_global):
    """The largest segment the select kernel takes (its candidate keys and flags fill LDS):
    180 x 180 patches = 32 candidates per thread in the global search; windows searched by
    the whole workgroup, no windows at all, windows searched by one wave each."""
    shape = _enc(wl.F32, batch=1, grid_h=180, grid_w=180, heads=2, head_dim=32, feat_dim=64,
                 win_rows=win, win_cols=win, keep_global=keep_global, keep_local=keep_local)
    inp, _, ref, info = pu.screened_encoder_case(shape, seed=9000, logit_gain=1.0)
    out = _run_encoder(shape, inp)
    print("max-segment", info, pu.check_encoder(shape, inp, ref, out, "max-segment"))
    # one more row of patches does not fit any more and is refused, not mis-computed
    too_big = dataclasses.replace(shape, grid_h=182)
    with pytest.raises(vb.VscanError) as e:
        vb.encoder_workspace_size(vb.encoder_desc(too_big))
    assert e.value.status == vb.VSCAN_ERR_UNSUPPORTED


# Shapes chosen so that, together with the cases above, every branch of the kernels' launch
# heuristics (register counts of the searches, window modes, tile forms, row widths) runs at
# least once.  Feature and head dimensions are kept small: the oracle stays cheap.
DISPATCH_ENCODER = {
    # select: one thread per token, 16 candidates per lane in the global wave
    "sel-900": _enc(grid_h=30, grid_w=30, heads=2, head_dim=16, feat_dim=32, win_rows=3,
                    win_cols=3, keep_global=20, keep_local=18),
    # select: one big window on a small segment (one wave searches up to 2048 window slots)
    "sel-one-window-400": _enc(grid_h=20, grid_w=20, heads=2, head_dim=16, feat_dim=32,
                               win_rows=1, win_cols=1, keep_global=0, keep_local=25),
    # select: large segment without windows, 4 and 16 candidates per thread
    "sel-global-1480": _enc(grid_h=40, grid_w=37, heads=2, head_dim=16, feat_dim=32,
                            win_rows=1, win_cols=1, keep_global=40, keep_local=0),
    "sel-global-5000": _enc(batch=1, grid_h=50, grid_w=100, heads=2, head_dim=16, feat_dim=32,
                            win_rows=1, win_cols=1, keep_global=40, keep_local=0),
    # select: mid-size windows searched by one wave each on a 4096-token segment
    "sel-wave-windows-4096": _enc(batch=1, grid_h=64, grid_w=64, heads=2, head_dim=16,
                                  feat_dim=32, win_rows=2, win_cols=4, keep_global=30,
                                  keep_local=24),
    # select: one window of 8100 tokens searched by the workgroup, 16 candidates per thread
    "sel-block-window-8100": _enc(batch=1, grid_h=90, grid_w=90, heads=2, head_dim=16,
                                  feat_dim=32, win_rows=1, win_cols=1, keep_global=20,
                                  keep_local=30),
    # select: small windows on the largest segment (32 candidates per thread, wave per window)
    "sel-small-windows-32400": _enc(wl.F32, batch=1, grid_h=180, grid_w=180, heads=2, head_dim=32,
                                    feat_dim=64, win_rows=12, win_cols=12, keep_global=20,
                                    keep_local=144),
    # select: one window over the largest segment (64 window slots per thread)
    "sel-one-window-32400": _enc(wl.F32, batch=1, grid_h=180, grid_w=180, heads=2, head_dim=32,
                                 feat_dim=64, win_rows=1, win_cols=1, keep_global=0,
                                 keep_local=32),
    # images pinned to XCDs with a batch that is not a multiple of eight (padding workgroups)
    "affine-batch-10": _enc(batch=10, grid_h=14, grid_w=14, heads=2, head_dim=16, feat_dim=96,
                            keep_global=12, keep_local=8),
    # merge: 4 and 8 pieces of a feature row per lane
    "merge-feat-2048": _enc(feat_dim=2048, heads=2),
    "merge-feat-4096": _enc(feat_dim=4096, heads=2),
    # mean-attention scoring: 256- and 512-byte head rows
    "mean-head-128": _enc(has_cls=0, score_mode=1, grid_h=12, grid_w=13, head_dim=128, heads=2),
    "mean-head-256": _enc(has_cls=0, score_mode=1, grid_h=11, grid_w=12, head_dim=256, heads=2),
    # similarity: the large-tile form in fp32
    "sim-large-tiles-f32": _enc(wl.F32, batch=8, grid_h=64, grid_w=64, heads=2, head_dim=16,
                                feat_dim=32, win_rows=1, win_cols=1, keep_global=512,
                                keep_local=0),
}


@pytest.mark.parametrize("name", sorted(DISPATCH_ENCODER))
def test_encoder_dispatch_coverage(name):
    shape = DISPATCH_ENCODER[name]
    # 144 window boundaries on flat scores never all clear the margin: peakier logits there
    gain = 2.0 if name == "sel-small-windows-32400" else 1.0
    inp, _, ref, info = pu.screened_encoder_batch(shape, seed=8000 + len(name), logit_gain=gain,
                                                  max_items=64 * shape.batch)
    out = _run_encoder(shape, inp)
    print(name, info, pu.check_encoder(shape, inp, ref, out, name))


DISPATCH_LLM = {
    # select: 16 candidates per thread
    "span-8000": _llm(batch=2, vis_len=8000, text=6, q_heads=1, kv_heads=1, head_dim=16,
                      hidden=16, keep=90),
    # scoring: few items with a long span are cut into chunks of 256 keys (ragged last chunk)
    "split-8x4500": _llm(batch=2, vis_len=4500, text=4, q_heads=8, kv_heads=1, head_dim=128,
                         hidden=16, keep=50),
    # ... also over the causal domain of several query positions, 12 query rows per kv head
    "split-causal-12x1500": _llm(batch=3, prefix=7, vis_len=1500, text=9, q_heads=8, kv_heads=2,
                                 n_query=3, head_dim=40, hidden=16, keep=400, softmax_domain=1),
    "f32-split-1x3000": _llm(wl.F32, batch=1, vis_len=3000, text=3, q_heads=2, kv_heads=2,
                             head_dim=24, hidden=16, keep=77),
    # scoring: logits of 17 rows x 2100 keys leave no LDS for the staging areas
    "unstaged-17x2100": _llm(batch=2, vis_len=2100, text=4, q_heads=17, kv_heads=1, head_dim=128,
                             hidden=16, keep=50),
    # scoring: 512-byte key rows with more than 16 query rows
    "f32-wide-many-rows": _llm(wl.F32, batch=2, vis_len=300, text=8, q_heads=8, kv_heads=2,
                               head_dim=128, hidden=16, keep=40, n_query=5),
}


@pytest.mark.parametrize("name", sorted(DISPATCH_LLM))
def test_llm_dispatch_coverage(name):
    shape = DISPATCH_LLM[name]
    inp, ref, info = pu.screened_llm_case(shape, seed=8500 + len(name), max_tries=48)
    print(name, info, pu.check_llm(shape, inp, ref, _run_llm(shape, inp), name))


# The 256 x 256 tile form of the similarity kernel (kept and dropped sets of a thousand rows
# and more, enough tiles for every CU), in its three tile orders.
SIM_LARGE = {
    # one image: every XCD works through its own block of tiles
    "one-image-xcd-blocks": _enc(batch=1, grid_h=96, grid_w=128, heads=2, head_dim=16, feat_dim=32,
                                 win_rows=1, win_cols=1, keep_global=4096, keep_local=0),
    # eight images: pinned to XCDs
    "eight-images-pinned": _enc(batch=8, grid_h=64, grid_w=80, heads=2, head_dim=16, feat_dim=40,
                                win_rows=1, win_cols=1, keep_global=1024, keep_local=0),
    # five kept tiles: not a multiple of the XCD block grid, tiles in launch order; ragged edges
    "two-images-launch-order": _enc(batch=2, grid_h=114, grid_w=128, heads=2, head_dim=16,
                                    feat_dim=32, win_rows=1, win_cols=1, keep_global=1270,
                                    keep_local=0),
    # rows of several 128-byte stages plus a ragged one (stages fetched straight into LDS, the
    # last through registers): 128 x 128 tiles, then 256 x 256 tiles, bf16 and fp32
    "staged-rows-400-bytes": _enc(batch=8, grid_h=64, grid_w=64, heads=2, head_dim=16, feat_dim=200,
                                  win_rows=1, win_cols=1, keep_global=512, keep_local=0),
    "staged-rows-288-bytes-f32": _enc(wl.F32, batch=1, grid_h=96, grid_w=128, heads=2, head_dim=16,
                                      feat_dim=72, win_rows=1, win_cols=1, keep_global=4096,
                                      keep_local=0),
}


@pytest.mark.parametrize("name", sorted(SIM_LARGE))
def test_encoder_similarity_large_tiles(name):
    shape = SIM_LARGE[name]
    inp, _, ref, info = pu.screened_encoder_case(shape, seed=8800 + len(name), logit_gain=1.0,
                                                 max_tries=2)
    out = _run_encoder(shape, inp)
    print(name, info, pu.check_encoder(shape, inp, ref, out, name))


def test_encoder_many_slots():
    """Enough kept slots in the batch that the merge gives every wave four slots in turn."""
    shape = _enc(batch=32, grid_h=24, grid_w=24, heads=2, feat_dim=72, win_rows=4, win_cols=4,
                 keep_global=128, keep_local=128)
    inp, _, ref, info = pu.screened_encoder_batch(shape, seed=4242, logit_gain=1.0)
    out = _run_encoder(shape, inp)
    print("many-slots", info, pu.check_encoder(shape, inp, ref, out, "many-slots"))


# ----------------------------------------------------------------------------
def test_config1_full():
    w = wl.config(1)
    inp, _, ref, info = pu.screened_encoder_case(w.encoder, w.seed)
    print("cfg1 encoder", info, pu.check_encoder(w.encoder, inp, ref, _run_encoder(w.encoder, inp)))
    inp, ref, info = pu.screened_llm_case(w.llm, w.seed)
    print("cfg1 llm", info, pu.check_llm(w.llm, inp, ref, _run_llm(w.llm, inp)))


@pytest.mark.parametrize("keep", [192, 128, 64])
def test_config2_full(keep):
    w = wl.config(2, sweep=keep)
    inp, _, ref, info = pu.screened_encoder_case(w.encoder, w.seed)
    print("cfg2 encoder", info, pu.check_encoder(w.encoder, inp, ref, _run_encoder(w.encoder, inp)))
    inp, ref, info = pu.screened_llm_case(w.llm, w.seed)
    print("cfg2 llm", info, pu.check_llm(w.llm, inp, ref, _run_llm(w.llm, inp)))


def test_config3_full():
    w = wl.config(3)
    inp, _, ref, info = pu.screened_encoder_case(w.encoder, w.seed)
    print("cfg3 encoder", info, pu.check_encoder(w.encoder, inp, ref, _run_encoder(w.encoder, inp)))
    inp, ref, info = pu.screened_llm_case(w.llm, w.seed)
    print("cfg3 llm", info, pu.check_llm(w.llm, inp, ref, _run_llm(w.llm, inp)))


def test_config6_video_full():
    w = wl.config(6)
    inp, _, ref, info = pu.screened_encoder_case(w.encoder, w.seed)
    print("cfg6 encoder", info, pu.check_encoder(w.encoder, inp, ref, _run_encoder(w.encoder, inp)))
    inp, ref, info = pu.screened_llm_case(w.llm, w.seed)
    print("cfg6 llm", info, pu.check_llm(w.llm, inp, ref, _run_llm(w.llm, inp)))


def test_config4_llm_full():
    w = wl.config(4)
    inp, ref, info = pu.screened_llm_case(w.llm, w.seed)
    print("cfg4 llm", info, pu.check_llm(w.llm, inp, ref, _run_llm(w.llm, inp)))


def test_config4_encoder_full():
    """Full size, the configuration's own seed.  64 window boundaries and one global boundary
    among 16384 flat column means: where one of them is closer than the margin, the validity
    check of check_encoder decides instead of bit-equality."""
    w = wl.config(4)
    shape = w.encoder
    inp = wl.encoder_inputs(shape, w.seed)
    ref = vo.encoder_reduce(shape, inp["q"], inp["k"], inp["x"])
    sg = ref["scores"].reshape(1, 1, -1)
    gap = pu.encoder_boundary_gap(shape, sg, sg)
    np.testing.assert_allclose(ref["scores"].sum(), 1.0, rtol=1e-9)
    out = _run_encoder(shape, inp)
    print("cfg4 encoder", {"gap": gap}, pu.check_encoder(shape, inp, ref, out, "cfg4"))


def test_config5_full():
    """Full-size stage-2 stress, all three budgets, every sequence against the oracle: scores
    element by element, kept indices bit-exact (valid where the oracle's boundary is closer
    than the margin), and hidden states, K and V against the order-preserving gather of the
    original rows under those indices (pure copies, evaluated on the device for all 32
    sequences; the oracle's own compaction is compared for the first two sequences)."""
    import torch
    base = wl.config(5)
    shape = base.llm
    B, S, V, vs = shape.batch, shape.seq_len, shape.vis_len, shape.vis_start
    keeps = (720, 288, 144)
    dev = {"q": torch.empty((B, shape.q_heads, shape.n_query, shape.head_dim), dtype=torch.bfloat16,
                            device="cuda"),
           "k": torch.empty((B, shape.kv_heads, S, shape.head_dim), dtype=torch.bfloat16,
                            device="cuda"),
           "hidden": torch.empty((B, S, shape.hidden), dtype=torch.bfloat16, device="cuda")}
    dev["v"] = torch.empty_like(dev["k"])
    host, s_ref = {}, np.empty((B, V))
    for b in range(B):
        item = wl.llm_item(shape, base.seed, b)
        for n in dev:
            dev[n][b].copy_(pu.to_device(item[n], shape.dtype))
        s_ref[b] = vo.llm_scores(item["q"][None], item["k"][None], vs, V)[0]
        if b < 2:
            host[b] = item
    orig = {n: dev[n].clone() for n in ("k", "v", "hidden")}

    for keep in keeps:
        sh = dataclasses.replace(shape, keep=keep)
        So = sh.seq_out
        for n in orig:
            dev[n].copy_(orig[n])
        out = vb.llm_prune(sh, dev["q"], dev["k"], dev["v"], dev["hidden"], want_scores=True)
        torch.cuda.synchronize()

        err = pu.check_scores(pu.to_host(out["scores"]), s_ref, f"cfg5 keep {keep}")
        kept_h = pu.to_host(out["kept_idx"])
        differing = pu.check_topk_rows(kept_h, vo.topk(s_ref, keep), s_ref, keep, f"cfg5 keep {keep}")

        kept = out["kept_idx"].long()
        rows = torch.cat([torch.arange(vs, device="cuda").expand(B, vs), vs + kept,
                          torch.arange(vs + V, S, device="cuda").expand(B, S - vs - V)], dim=1)
        assert rows.shape == (B, So)
        want_h = torch.gather(orig["hidden"], 1, rows[:, :, None].expand(B, So, sh.hidden))
        assert torch.equal(out["hidden"], want_h)
        idx = rows[:, None, :, None].expand(B, sh.kv_heads, So, sh.head_dim)
        assert torch.equal(out["k"], torch.gather(orig["k"], 2, idx))
        assert torch.equal(out["v"], torch.gather(orig["v"], 2, idx))

        one = dataclasses.replace(sh, batch=1)
        for b in host:
            for n in ("k", "v", "hidden"):
                want = vo.compact(host[b][n][None], kept_h[b:b + 1], vs, V)
                assert np.array_equal(pu.to_host(out[n][b:b + 1]), want), (keep, b, n)
        print("cfg5 keep", keep, {"score_rel_err": err, "rows_valid_not_identical": differing},
              flush=True)
