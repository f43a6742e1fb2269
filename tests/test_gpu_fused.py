"""GPU parity of stage 2 scored from hidden states and projection weights (Eq. 5 as written)
against the CPU oracle's plain definition.  Rules and tolerances: tests/parity_utils.py."""
import dataclasses

import numpy as np
import pytest

from oracle import vscan_oracle as vo
from paper_2505_22654_amd import binding as vb
from paper_2505_22654_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu


def _run(shape, inp):
    import torch
    h = pu.to_device(inp["hidden"], shape.dtype)
    wq = pu.to_device(inp["w_q"], shape.dtype)
    wkt = pu.to_device(np.ascontiguousarray(inp["w_k"].T), shape.dtype)
    out = vb.llm_prune_fused(shape, h, wq, wkt, want_scores=True)
    torch.cuda.synchronize()
    return out


def _shape(**kw):
    base = dict(dtype=wl.BF16, batch=2, prefix=5, vis_len=150, text=9, n_query=1, q_heads=8,
                kv_heads=8, head_dim=64, hidden=512, keep=40)
    base.update(kw)
    return wl.LlmShape(**base)


SMALL_FUSED = {
    # several 128-row tiles with a ragged tail; hidden size not a multiple of the 64-element chunk
    "ragged-tiles": _shape(batch=3, vis_len=300, hidden=520, keep=100),
    "in-place": _shape(in_place=1),
    "all-keys": _shape(softmax_domain=1, prefix=37, text=21),
    # all keys and several query positions: each position's row is causal
    "all-keys-queries": _shape(softmax_domain=1, n_query=3, q_heads=8, kv_heads=4, text=11),
    # grouped heads and several query positions: 24 query rows
    "gqa-queries": _shape(q_heads=8, kv_heads=2, n_query=3, head_dim=32, hidden=256),
    # more query rows than one 128-row tile of the plane operand
    "many-rows": _shape(q_heads=16, kv_heads=4, n_query=9, head_dim=40, hidden=320, vis_len=200,
                        text=12, keep=60),
    # 33..64 query rows (two 32-row tiles per workgroup)
    "two-row-tiles": _shape(q_heads=12, kv_heads=12, n_query=4, head_dim=24, hidden=264),
    # long rows and few output tiles: the contraction axis is split over workgroups
    "split-axis": _shape(batch=1, hidden=4096, q_heads=4, kv_heads=2, head_dim=128, vis_len=70,
                         keep=11),
    # key domains of every softmax form: up to 1024, up to 4096, longer
    "domain-1k": _shape(batch=1, vis_len=700, keep=200, hidden=128, q_heads=4, kv_heads=4, head_dim=32),
    "domain-4k": _shape(batch=1, vis_len=2500, keep=700, hidden=64, q_heads=2, kv_heads=1, head_dim=32),
    # many rows of a long domain
    "domain-4k-many-rows": _shape(batch=8, vis_len=1100, keep=40, hidden=64, q_heads=16, kv_heads=4,
                                  head_dim=16, n_query=8),
    "domain-long": _shape(batch=1, vis_len=4300, keep=1000, hidden=64, q_heads=2, kv_heads=2,
                          head_dim=32, n_query=2),
    "domain-longest": _shape(batch=1, vis_len=17000, keep=3000, hidden=64, q_heads=1, kv_heads=1,
                             head_dim=32),
    # eight or more sequences: a sequence's workgroups stay on one XCD
    "nine-sequences": _shape(batch=9, vis_len=140, keep=30, hidden=128, q_heads=4, kv_heads=2,
                             head_dim=32),
    "one-visual-token": _shape(vis_len=1, keep=1),
    "keep-nothing": _shape(keep=0),
    "keep-everything": _shape(keep=150),
    "head-dim-8": _shape(head_dim=8, hidden=64, q_heads=3, kv_heads=1),
}


@pytest.mark.parametrize("name", sorted(SMALL_FUSED))
def test_fused_small(name):
    shape = SMALL_FUSED[name]
    inp, ref, info = pu.screened_fused_case(shape, 9100 + sorted(SMALL_FUSED).index(name) * 31)
    print("case", name, info, flush=True)
    out = _run(shape, inp)
    print(name, pu.check_fused(shape, ref, out, name, hidden=inp["hidden"]))


FUSED_F32 = {
    # fp32 hidden states and weights: the same chain on fp32 matrix instructions, q and the
    # hidden-space query carried as fp32 values instead of bf16 planes
    "f32": _shape(dtype=wl.F32),
    "f32-ragged-tiles": _shape(dtype=wl.F32, batch=3, vis_len=300, hidden=520, keep=100),
    "f32-in-place": _shape(dtype=wl.F32, in_place=1),
    "f32-all-keys-queries": _shape(dtype=wl.F32, softmax_domain=1, n_query=3, q_heads=8, kv_heads=4,
                                   text=11),
    "f32-many-rows": _shape(dtype=wl.F32, q_heads=16, kv_heads=4, n_query=9, head_dim=40, hidden=320,
                            vis_len=200, text=12, keep=60),
    "f32-split-axis": _shape(dtype=wl.F32, batch=1, hidden=2048, q_heads=4, kv_heads=2, head_dim=128,
                             vis_len=70, keep=11),
}


@pytest.mark.parametrize("name", sorted(FUSED_F32))
def test_fused_fp32(name):
    shape = FUSED_F32[name]
    inp, ref, info = pu.screened_fused_case(shape, 9300 + sorted(FUSED_F32).index(name) * 29)
    print("case", name, info, flush=True)
    out = _run(shape, inp)
    print(name, pu.check_fused(shape, ref, out, name, hidden=inp["hidden"]))


def test_fused_agrees_with_projected_path():
    """The same selection as vscan_llm_prune fed with q and k projected on the host (fp64, rounded
    to fp32): two routes to Eq. 5 through different kernels."""
    import torch
    shape = _shape(dtype=wl.F32, batch=2, vis_len=260, keep=77, hidden=384)
    bshape = dataclasses.replace(shape, dtype=wl.BF16)
    inp, ref, info = pu.screened_fused_case(bshape, 9900)
    print("case", info, flush=True)
    out = _run(bshape, inp)
    x = inp["hidden"].astype(np.float64)
    B, S, _ = x.shape
    q = (x[:, S - 1:] @ inp["w_q"].astype(np.float64).T).reshape(B, 1, 8, 64).transpose(0, 2, 1, 3)
    k = (x @ inp["w_k"].astype(np.float64).T).reshape(B, S, 8, 64).transpose(0, 2, 1, 3)
    dev = [pu.to_device(np.ascontiguousarray(a, dtype=np.float32), wl.F32)
           for a in (q, k, k, inp["hidden"])]
    proj = vb.llm_prune(shape, *dev, want_scores=True)
    torch.cuda.synchronize()
    assert torch.equal(proj["kept_idx"], out["kept_idx"])
    np.testing.assert_allclose(pu.to_host(out["scores"]), pu.to_host(proj["scores"]), rtol=4e-5)


def test_fused_runs_are_bit_reproducible():
    import torch
    shape = SMALL_FUSED["split-axis"]
    inp, _, _ = pu.screened_fused_case(shape, 9300)
    a, b = _run(shape, inp), _run(shape, inp)
    assert torch.equal(a["kept_idx"], b["kept_idx"])
    assert torch.equal(a["scores"], b["scores"])


def test_fused_config2_shape():
    """The stage-2 shape of the headline configuration (16 sequences, 192 visual tokens, 32 heads
    of 128, hidden 4096), every sequence checked against the oracle."""
    shape = wl.config(2).llm
    inp, ref, info = pu.screened_fused_case(shape, 9500, max_tries=4)
    print("case", info, flush=True)
    out = _run(shape, inp)
    print("cfg2 stage-2 shape", pu.check_fused(shape, ref, out, "cfg2 fused", hidden=inp["hidden"]))


def test_fused_more_sequences_than_one_row_tile():
    """33 sequences of 4 query positions: 132 query rows in the query projection (its largest
    tile shape), 33 rows per kv head in the hidden-space step."""
    shape = _shape(batch=33, n_query=4, vis_len=90, keep=20, hidden=128, q_heads=4, kv_heads=4,
                   head_dim=16, prefix=3, text=6)
    inp, ref, info = pu.screened_fused_case(shape, 9650)
    print("case", info, flush=True)
    print(pu.check_fused(shape, ref, _run(shape, inp), "33 sequences", hidden=inp["hidden"]))
    shape = dataclasses.replace(shape, batch=20)      # 80 query rows: the 128-row tile shape
    inp, ref, info = pu.screened_fused_case(shape, 9660)
    print("case", info, flush=True)
    print(pu.check_fused(shape, ref, _run(shape, inp), "20 sequences", hidden=inp["hidden"]))


def test_fused_config5_full():
    """Full-size stage-2 stress shape (32 sequences, 2880 visual tokens, 8 query positions = 256
    query rows, hidden 4096), in place, all three budgets, every sequence against the oracle:
    scores element by element, kept indices bit-exact (valid where the oracle's boundary is
    closer than the margin), hidden states against the order-preserving gather of the original
    rows under those indices (on the device for all sequences; the oracle's own compaction for
    the first two)."""
    import torch
    base = wl.config(5)
    shape = base.llm
    B, S, V, vs = shape.batch, shape.seq_len, shape.vis_len, shape.vis_start
    keeps = (720, 288, 144)
    w = wl.llm_weights(shape, base.seed)
    wq = pu.to_device(w["w_q"], wl.BF16)
    wkt = pu.to_device(np.ascontiguousarray(w["w_k"].T), wl.BF16)
    hidden = torch.empty((B, S, shape.hidden), dtype=torch.bfloat16, device="cuda")
    host, s_ref = {}, np.empty((B, V))
    for b in range(B):
        item = wl.llm_item(shape, base.seed, b)["hidden"]
        hidden[b].copy_(pu.to_device(item, wl.BF16))
        s_ref[b] = vo.llm_scores_from_hidden(item[None], w["w_q"], w["w_k"], vs, V, shape.n_query,
                                             shape.q_heads, shape.kv_heads, shape.head_dim)[0]
        if b < 2:
            host[b] = item
    orig = hidden.clone()

    for keep in keeps:
        sh = dataclasses.replace(shape, keep=keep)
        So = sh.seq_out
        hidden.copy_(orig)
        out = vb.llm_prune_fused(sh, hidden, wq, wkt, want_scores=True)
        torch.cuda.synchronize()
        err = pu.check_scores(pu.to_host(out["scores"]), s_ref, f"cfg5 fused keep {keep}")
        kept_h = pu.to_host(out["kept_idx"])
        differing = pu.check_topk_rows(kept_h, vo.topk(s_ref, keep), s_ref, keep,
                                       f"cfg5 fused keep {keep}")
        kept = out["kept_idx"].long()
        rows = torch.cat([torch.arange(vs, device="cuda").expand(B, vs), vs + kept,
                          torch.arange(vs + V, S, device="cuda").expand(B, S - vs - V)], dim=1)
        assert rows.shape == (B, So)
        want_h = torch.gather(orig, 1, rows[:, :, None].expand(B, So, sh.hidden))
        assert torch.equal(out["hidden"], want_h)
        for b in host:
            ref_h = vo.compact(host[b][None], kept_h[b:b + 1], vs, V)
            assert np.array_equal(pu.to_host(out["hidden"][b:b + 1]), ref_h), (keep, b)
        print("cfg5 fused keep", keep, {"score_rel_err": err, "rows_valid_not_identical": differing},
              flush=True)


RAGGED_SEQS = [
    # (prefix, vis_len, text, keep): long and short spans, nothing kept, everything kept, a span
    # shorter than one tile, the longest sequence not the one with the longest span
    (35, 600, 70, 200), (3, 5, 9, 2), (0, 333, 41, 0), (12, 257, 300, 257), (7, 700, 13, 1),
    (20, 64, 20, 63), (1, 130, 4, 30), (9, 40, 6, 11), (2, 300, 3, 150),
]


@pytest.mark.parametrize("variant", ["plain", "in-place-queries", "all-keys-gqa"])
def test_fused_ragged(variant):
    """Per-sequence lengths, spans and budgets in one call, each sequence against the oracle run
    on that sequence alone (nine sequences: each stays on one XCD)."""
    import torch
    base = {
        "plain": _shape(hidden=256, q_heads=4, kv_heads=4, head_dim=32),
        "in-place-queries": _shape(in_place=1, n_query=2, hidden=136, q_heads=4, kv_heads=4, head_dim=32),
        "all-keys-gqa": _shape(softmax_domain=1, n_query=3, q_heads=8, kv_heads=2, head_dim=16,
                               hidden=128),
    }[variant]
    seqs = [(p, v, max(t, base.n_query), k) for p, v, t, k in RAGGED_SEQS]
    caps, meta, inp, refs = pu.ragged_fused_case(base, seqs, seed=9900 + len(variant))
    h, wq = pu.to_device(inp["hidden"], wl.BF16), pu.to_device(inp["w_q"], wl.BF16)
    wkt = pu.to_device(np.ascontiguousarray(inp["w_k"].T), wl.BF16)
    out = vb.llm_prune_fused_ragged(caps, meta, h, wq, wkt, want_scores=True)
    torch.cuda.synchronize()
    print(variant, pu.check_fused_ragged(caps, meta, inp, refs, out, caps.in_place, variant))


def test_fused_ragged_matches_uniform():
    import torch
    shape = _shape(batch=4, prefix=9, vis_len=400, text=33, keep=100, n_query=2, hidden=128,
                   q_heads=4, kv_heads=2, head_dim=32)
    inp, ref, info = pu.screened_fused_case(shape, 9950)
    dev = lambda: (pu.to_device(inp["hidden"], wl.BF16), pu.to_device(inp["w_q"], wl.BF16),
                   pu.to_device(np.ascontiguousarray(inp["w_k"].T), wl.BF16))
    uni = vb.llm_prune_fused(shape, *dev(), want_scores=True)
    meta = [(shape.seq_len, shape.vis_start, shape.vis_len, shape.keep)] * shape.batch
    rag = vb.llm_prune_fused_ragged(shape, meta, *dev(), want_scores=True)
    torch.cuda.synchronize()
    assert torch.equal(uni["kept_idx"], rag["kept_idx"]) and torch.equal(uni["scores"], rag["scores"])
    assert torch.equal(uni["hidden"], rag["hidden"][:, :shape.seq_out])
    print("ragged == uniform", info, pu.check_fused(shape, ref, uni, "uniform", hidden=inp["hidden"]))


# ---- stage 1 scored from the layer's input rows and projection weights -------------------------

def _run_encoder(shape, inp, loc=None):
    import torch
    dev = lambda a: pu.to_device(a, shape.dtype)
    triple = lambda d: (dev(d["hidden"]), dev(d["w_q"]), dev(np.ascontiguousarray(d["w_k"].T)))
    h, wq, wkt = triple(inp)
    out = vb.encoder_reduce_fused(shape, h, wq, wkt, dev(inp["x"]),
                                  local=None if loc is None else triple(loc), want_assign=True,
                                  want_scores=True)
    torch.cuda.synchronize()
    return out


def _enc(**kw):
    base = dict(dtype=wl.BF16, batch=2, n_segments=1, grid_h=12, grid_w=12, has_cls=1, score_mode=0,
                heads=4, head_dim=32, feat_dim=128, win_rows=2, win_cols=2, keep_global=10,
                keep_local=8)
    base.update(kw)
    return wl.EncoderShape(**base)


FUSED_ENCODER = {
    # 36 segments: more than one 32-row tile of [CLS] queries
    "many-images": _enc(batch=12, n_segments=3, grid_h=6, grid_w=6, heads=2, head_dim=16,
                        feat_dim=64, win_rows=1, win_cols=1, keep_global=5, keep_local=0),
    "ragged": _enc(batch=3, n_segments=2, grid_h=13, grid_w=11, heads=3, head_dim=40, feat_dim=200,
                   win_rows=3, win_cols=2, keep_global=17, keep_local=13),
    "all-keys": _enc(softmax_domain=1, keep_global=30, keep_local=16),
    "global-only": _enc(keep_local=0, keep_global=21),
    "many-segments": _enc(batch=2, n_segments=5, grid_h=8, grid_w=8, keep_global=6, keep_local=4),
}


@pytest.mark.parametrize("name", sorted(FUSED_ENCODER))
def test_fused_encoder_small(name):
    shape = FUSED_ENCODER[name]
    inp, _, ref, info = pu.screened_encoder_fused_case(shape, 9700 + sorted(FUSED_ENCODER).index(name) * 17)
    print("case", name, info, flush=True)
    out = _run_encoder(shape, inp)
    print(name, pu.check_encoder(shape, inp, ref, out, name))


def test_fused_encoder_local_scan_from_shallow_layer():
    shape = _enc(batch=2, grid_h=12, grid_w=12, keep_global=14, keep_local=12)
    inp, loc, ref, info = pu.screened_encoder_fused_case(shape, 9800, with_local=True)
    print("case", info, flush=True)
    assert not np.array_equal(ref["scores"], ref["scores_local"])
    out = _run_encoder(shape, inp, loc)
    print(pu.check_encoder(shape, inp, ref, out, "fused encoder, shallow-layer local scan"))


def test_fused_encoder_rejects_wide_mean_heads():
    with pytest.raises(vb.VscanError) as e:
        vb.encoder_fused_workspace_size(vb.encoder_desc(_enc(has_cls=0, score_mode=1, head_dim=136)))
    assert e.value.status == vb.VSCAN_ERR_UNSUPPORTED


@pytest.mark.parametrize("mode", ["cls", "cls-all-keys", "mean", "mean-with-cls"])
def test_fused_encoder_fp32(mode):
    shape = {"cls": _enc(dtype=wl.F32),
             "cls-all-keys": _enc(dtype=wl.F32, softmax_domain=1, batch=3, n_segments=2, grid_h=13,
                                  grid_w=11, heads=3, head_dim=40, feat_dim=200, win_rows=3, win_cols=2,
                                  keep_global=17, keep_local=13),
             "mean": _enc(dtype=wl.F32, has_cls=0, score_mode=1, grid_h=11, grid_w=13, heads=3,
                          head_dim=24, feat_dim=96),
             "mean-with-cls": _enc(dtype=wl.F32, has_cls=1, score_mode=1, softmax_domain=1)}[mode]
    inp, _, ref, info = pu.screened_encoder_fused_case(shape, 9990, max_tries=6)
    print("case", mode, info, flush=True)
    out = _run_encoder(shape, inp)
    print(mode, pu.check_encoder(shape, inp, ref, out, "fused encoder fp32 " + mode))


FUSED_ENCODER_MEAN = {
    # no [CLS] row (the encoder the mean-attention sentence is about), ragged grid and head size
    "no-cls": _enc(has_cls=0, score_mode=1, batch=2, n_segments=2, grid_h=13, grid_w=11, heads=3,
                   head_dim=40, feat_dim=200, win_rows=3, win_cols=2, keep_global=17, keep_local=13),
    # a [CLS] row that only takes part as a key
    "cls-all-keys": _enc(has_cls=1, score_mode=1, softmax_domain=1, keep_global=30, keep_local=16),
    "cls-patch-keys": _enc(has_cls=1, score_mode=1, grid_h=9, grid_w=14, heads=2, head_dim=64),
    # more tokens than one 256-row tile of the projection, 128-wide heads (the fp32 limit)
    "many-rows-wide-heads": _enc(has_cls=0, score_mode=1, batch=3, n_segments=2, grid_h=16,
                                 grid_w=15, heads=2, head_dim=128, feat_dim=256, keep_global=12,
                                 keep_local=8),
}


@pytest.mark.parametrize("name", sorted(FUSED_ENCODER_MEAN))
def test_fused_encoder_mean_attention(name):
    """Stage 1 scored by mean attention received, from hidden states and projection weights."""
    shape = FUSED_ENCODER_MEAN[name]
    inp, _, ref, info = pu.screened_encoder_fused_case(
        shape, 9900 + sorted(FUSED_ENCODER_MEAN).index(name) * 13, max_tries=6)
    print("case", name, info, flush=True)
    out = _run_encoder(shape, inp)
    print(name, pu.check_encoder(shape, inp, ref, out, name))


def test_fused_encoder_mean_attention_with_shallow_layer():
    shape = _enc(has_cls=0, score_mode=1, batch=2, grid_h=12, grid_w=12, keep_global=14, keep_local=12)
    inp, loc, ref, info = pu.screened_encoder_fused_case(shape, 9950, with_local=True, max_tries=6)
    print("case", info, flush=True)
    out = _run_encoder(shape, inp, loc)
    print(pu.check_encoder(shape, inp, ref, out, "fused encoder, mean attention, shallow-layer local scan"))


def test_fused_encoder_mean_attention_agrees_with_projected_path():
    """The same scores through the other route: Q and K projected on the host (rounded to fp32)
    and handed to vscan_encoder_reduce in mean mode."""
    import torch
    shape = _enc(has_cls=0, score_mode=1, batch=2, grid_h=10, grid_w=9, heads=3, head_dim=24, feat_dim=96)
    inp = wl.encoder_hidden_inputs(shape, 9960)
    out = _run_encoder(shape, inp)
    x = inp["hidden"].astype(np.float64)
    B, C, S, D = x.shape
    H, dh = shape.heads, shape.head_dim
    q = (x @ inp["w_q"].astype(np.float64).T).reshape(B, C, S, H, dh).transpose(0, 1, 3, 2, 4)
    k = (x @ inp["w_k"].astype(np.float64).T).reshape(B, C, S, H, dh).transpose(0, 1, 3, 2, 4)
    f32 = dataclasses.replace(shape, dtype=wl.F32)
    other = vb.encoder_reduce(f32, pu.to_device(np.ascontiguousarray(q, dtype=np.float32), wl.F32),
                              pu.to_device(np.ascontiguousarray(k, dtype=np.float32), wl.F32),
                              pu.to_device(inp["x"].astype(np.float32), wl.F32), want_scores=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(pu.to_host(out["scores"]), pu.to_host(other["scores"]), rtol=2e-5)


def test_fused_encoder_config2_shape():
    """The stage-1 shape of the headline configuration (16 images, 576 patches + [CLS], 16 heads
    of 64, 1024 features), every image checked against the oracle."""
    shape = wl.config(2).encoder
    inp, _, ref, info = pu.screened_encoder_fused_case(shape, 9850, max_tries=6)
    print("case", info, flush=True)
    out = _run_encoder(shape, inp)
    print("cfg2 stage-1 shape", pu.check_encoder(shape, inp, ref, out, "cfg2 fused encoder"))


def test_both_forms_replay_from_a_captured_graph():
    """The entry points allocate nothing, never synchronise and clear their own scratch words, so
    a call sequence can be captured once and replayed: three replays on fresh inputs, with eager
    work in between, each bit-identical to the eager calls on the same inputs."""
    import torch
    enc = _enc(batch=3, n_segments=2, grid_h=13, grid_w=11, heads=3, head_dim=40, feat_dim=200,
               win_rows=3, win_cols=2, keep_global=17, keep_local=13)
    llm = _shape(batch=3, vis_len=300, hidden=264, keep=100, n_query=2, q_heads=8, kv_heads=4,
                 head_dim=32)

    def host(trial):
        e = wl.encoder_inputs(enc, 4100 + trial, 0.25)
        l = wl.llm_inputs(llm, 4200 + trial)
        w = wl.llm_weights(llm, 4200 + trial)
        return {"eq": e["q"], "ek": e["k"], "ex": e["x"], "lq": l["q"], "lk": l["k"], "lv": l["v"],
                "lh": l["hidden"], "wq": w["w_q"], "wkt": np.ascontiguousarray(w["w_k"].T)}

    dev = {n: pu.to_device(a, wl.BF16) for n, a in host(0).items()}

    def outputs():
        z = lambda shape, dt: torch.zeros(shape, dtype=dt, device="cuda")
        bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
        So = llm.seq_out
        return ({"kept_idx": z((enc.batch, enc.keep), i32), "merged": z((enc.batch, enc.keep, enc.feat_dim), bf),
                 "assign": z((enc.batch, enc.tokens_per_image), i32),
                 "scores": z((enc.batch, enc.tokens_per_image), f32)},
                {"kept_idx": z((llm.batch, llm.keep), i32), "scores": z((llm.batch, llm.vis_len), f32),
                 "k": z((llm.batch, llm.kv_heads, So, llm.head_dim), bf),
                 "v": z((llm.batch, llm.kv_heads, So, llm.head_dim), bf),
                 "hidden": z((llm.batch, So, llm.hidden), bf)},
                {"kept_idx": z((llm.batch, llm.keep), i32), "scores": z((llm.batch, llm.vis_len), f32),
                 "hidden": z((llm.batch, So, llm.hidden), bf)})

    ws = [torch.empty(n, dtype=torch.uint8, device="cuda") for n in (
        vb.encoder_workspace_size(vb.encoder_desc(enc)), vb.llm_workspace_size(vb.llm_desc(llm)),
        vb.llm_fused_workspace_size(vb.llm_desc(llm)))]

    def calls(outs):
        vb.encoder_reduce(enc, dev["eq"], dev["ek"], dev["ex"], want_assign=True, want_scores=True,
                          workspace=ws[0], out=outs[0])
        vb.llm_prune(llm, dev["lq"], dev["lk"], dev["lv"], dev["lh"], want_scores=True,
                     workspace=ws[1], out=outs[1])
        vb.llm_prune_fused(llm, dev["lh"], dev["wq"], dev["wkt"], want_scores=True,
                           workspace=ws[2], out=outs[2])

    graph_out = outputs()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        calls(graph_out)                      # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        calls(graph_out)
    torch.cuda.synchronize()

    for trial in range(1, 4):
        for n, a in host(trial).items():
            dev[n].copy_(pu.to_device(a, wl.BF16))
        for o in graph_out:                   # stale results must not pass for fresh ones
            for t in o.values():
                if torch.is_tensor(t):
                    t.zero_()
        g.replay()
        torch.cuda.synchronize()
        eager_out = outputs()
        calls(eager_out)
        torch.cuda.synchronize()
        for got, want in zip(graph_out, eager_out):
            for name in want:
                if torch.is_tensor(want[name]) and name != "workspace":
                    assert torch.equal(got[name], want[name]), (trial, name)
        assert int(eager_out[1]["kept_idx"].max()) > 0
