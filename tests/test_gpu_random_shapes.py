"""GPU parity on randomly drawn small shapes (fixed generator seed, so the same shapes every
run): every entry point against the oracle, within the documented limits of the kernels.  No shape
is skipped: without a clear selection boundary the validity check decides."""
import numpy as np
import pytest

from paper_2505_22654_amd import binding as vb
from paper_2505_22654_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu

N_SHAPES = 64


def _sync():
    import torch
    torch.cuda.synchronize()


def _encoder_shape(r, fused=False):
    mean = r.random() < 0.3      # the entry points that score from hidden states take both modes
    has_cls = 1 if not mean else int(r.integers(0, 2))
    dtype = wl.BF16 if r.random() < 0.6 else wl.F32    # every entry point takes both
    gh, gw = int(r.integers(3, 19)), int(r.integers(3, 19))
    wr, wc = int(r.integers(1, min(gh, 4) + 1)), int(r.integers(1, min(gw, 4) + 1))
    n, w = gh * gw, wr * wc
    smallest_window = (gh // wr) * (gw // wc)
    kw = int(r.integers(0, min(smallest_window, 4) + 1))
    keep_local = kw * w + int(r.integers(0, w))                 # a remainder goes to the global scan
    keep_local = min(keep_local, n - 1)
    keep_global = int(r.integers(0 if keep_local else 1, max(1, min(n - keep_local, 40)) + 1))
    return wl.EncoderShape(
        dtype=dtype, batch=int(r.integers(1, 4)), n_segments=int(r.integers(1, 4)), grid_h=gh,
        grid_w=gw, has_cls=has_cls, score_mode=int(mean), heads=int(r.integers(1, 6)),
        head_dim=8 * int(r.integers(1, 11)), feat_dim=8 * int(r.integers(2, 34)), win_rows=wr,
        win_cols=wc, keep_global=keep_global, keep_local=keep_local,
        softmax_domain=int(r.integers(0, 2)) if has_cls else 0)


def _llm_shape(r, fused=False):
    kv = int(r.integers(1, 5))
    group = int(r.integers(1, 4))
    tq = int(r.integers(1, 4))
    vis = int(r.integers(1, 400))
    return wl.LlmShape(
        dtype=wl.BF16 if r.random() < 0.6 else wl.F32, batch=int(r.integers(1, 6)),
        prefix=int(r.integers(0, 10)), vis_len=vis, text=tq + int(r.integers(0, 20)), n_query=tq,
        q_heads=kv * group, kv_heads=kv, head_dim=8 * int(r.integers(1, 17)),
        hidden=8 * int(r.integers(1, 34)), keep=int(r.integers(0, vis + 1)),
        in_place=int(r.integers(0, 2)), softmax_domain=int(r.integers(0, 2)))


def _sweep(draw, screen, run, check):
    """Every drawn shape runs.  A shape whose first seeds leave no clear selection boundary is
    taken with the widest-gap seed and judged by the validity check (parity_utils)."""
    r = np.random.default_rng(20250522)
    unclear = 0
    for i in range(N_SHAPES):
        shape = draw(r)
        case = screen(shape, 31000 + 97 * i)
        unclear += "margin" in case[-1]
        print("shape", i, shape, case[-1], flush=True)
        check(shape, case, run(shape, case))
    print(f"{N_SHAPES} shapes run, {unclear} of them without a clear boundary", flush=True)


def test_random_encoder_shapes():
    def run(shape, case):
        inp = case[0]
        q, k, x = (pu.to_device(inp[n], shape.dtype) for n in ("q", "k", "x"))
        out = vb.encoder_reduce(shape, q, k, x, want_assign=True, want_scores=True)
        _sync()
        return out
    _sweep(_encoder_shape, lambda s, seed: pu.screened_encoder_case(s, seed, 0.25, max_tries=4), run,
           lambda s, case, out: pu.check_encoder(s, case[0], case[2], out, str(s)))


def test_random_llm_shapes():
    def run(shape, case):
        inp = case[0]
        q, k, v, h = (pu.to_device(inp[n], shape.dtype) for n in ("q", "k", "v", "hidden"))
        out = vb.llm_prune(shape, q, k, v, h, want_scores=True)
        _sync()
        return out
    _sweep(_llm_shape, lambda s, seed: pu.screened_llm_case(s, seed, max_tries=4), run,
           lambda s, case, out: pu.check_llm(s, case[0], case[1], out, str(s)))


def test_random_fused_llm_shapes():
    def run(shape, case):
        inp = case[0]
        h, wq = pu.to_device(inp["hidden"], shape.dtype), pu.to_device(inp["w_q"], shape.dtype)
        wkt = pu.to_device(np.ascontiguousarray(inp["w_k"].T), shape.dtype)
        out = vb.llm_prune_fused(shape, h, wq, wkt, want_scores=True)
        _sync()
        return out
    _sweep(lambda r: _llm_shape(r, fused=True),
           lambda s, seed: pu.screened_fused_case(s, seed, max_tries=4), run,
           lambda s, case, out: pu.check_fused(s, case[1], out, str(s), hidden=case[0]["hidden"]))


def test_random_fused_encoder_shapes():
    def run(shape, case):
        inp = case[0]
        dev = lambda a: pu.to_device(a, shape.dtype)
        out = vb.encoder_reduce_fused(shape, dev(inp["hidden"]), dev(inp["w_q"]),
                                      dev(np.ascontiguousarray(inp["w_k"].T)), dev(inp["x"]),
                                      want_assign=True, want_scores=True)
        _sync()
        return out
    _sweep(lambda r: _encoder_shape(r, fused=True),
           lambda s, seed: pu.screened_encoder_fused_case(s, seed, 0.25, max_tries=4), run,
           lambda s, case, out: pu.check_encoder(s, case[0], case[2], out, str(s)))


def test_random_wide_rows_with_clustered_features():
    """Feature rows of 96 to 300 16-byte pieces (from 128 on the merge adds them as two column
    halves) drawn around a few prototypes, so that groups of a few dozen to a few hundred members
    occur: shared groups, groups longer than a slot's list, ragged column halves."""
    import torch
    from oracle import vscan_oracle as vo
    r = np.random.default_rng(20250523)
    largest = 0
    for i in range(16):
        dtype = wl.BF16 if r.random() < 0.6 else wl.F32
        pieces = int(r.choice([96, 127, 128, 129, 130, 160, 191, 192, 200, 256, 257, 300]))
        if dtype == wl.F32:
            pieces += pieces % 2  # feature rows are whole multiples of 8 elements
        gh, gw = int(r.integers(8, 45)), int(r.integers(8, 45))
        wr, wc = int(r.integers(1, 4)), int(r.integers(1, 4))
        shape = wl.EncoderShape(
            dtype=dtype, batch=int(r.integers(1, 4)), n_segments=int(r.integers(1, 3)), grid_h=gh,
            grid_w=gw, has_cls=1, score_mode=0, heads=2, head_dim=16,
            feat_dim=pieces * (8 if dtype == wl.BF16 else 4), win_rows=wr, win_cols=wc,
            keep_global=int(r.integers(1, max(2, gh * gw // 8))),
            keep_local=int(r.integers(0, 4)) * wr * wc, softmax_domain=0)
        inp = wl.encoder_inputs(shape, 9000 + i)
        T = shape.n_segments * gh * gw
        protos = r.standard_normal((int(r.integers(2, 9)), shape.feat_dim)).astype(np.float32)
        which = r.integers(0, len(protos), size=(shape.batch, T))
        x = protos[which] + 0.05 * r.standard_normal((shape.batch, T, shape.feat_dim)).astype(np.float32)
        inp["x"] = wl.round_to_bf16(x) if dtype == wl.BF16 else x
        ref = vo.encoder_reduce(shape, inp["q"], inp["k"], inp["x"])
        largest = max(largest, max(int(np.bincount(ref["assign"][b], minlength=shape.keep).max())
                                   for b in range(shape.batch)))
        q, k, xd = (pu.to_device(inp[n], shape.dtype) for n in ("q", "k", "x"))
        out = vb.encoder_reduce(shape, q, k, xd, want_assign=True, want_scores=True)
        torch.cuda.synchronize()
        print("shape", i, shape, pu.check_encoder(shape, inp, ref, out, str(shape)), flush=True)
    assert largest > 128, largest  # the draw covers groups longer than a slot's list


def test_random_encoder_shapes_with_shallow_layer_pair():
    def run(shape, case):
        inp, loc = case[0], case[1]
        q, k, x = (pu.to_device(inp[n], shape.dtype) for n in ("q", "k", "x"))
        ql, kl = pu.to_device(loc["q"], shape.dtype), pu.to_device(loc["k"], shape.dtype)
        out = vb.encoder_reduce(shape, q, k, x, ql, kl, want_assign=True, want_scores=True)
        _sync()
        return out
    _sweep(_encoder_shape,
           lambda s, seed: pu.screened_encoder_case(s, seed, 0.25, with_local=True, max_tries=4), run,
           lambda s, case, out: pu.check_encoder(s, case[0], case[2], out, str(s)))


def _ragged_draw(r, fused):
    base = _llm_shape(r, fused)
    seqs = []
    for _ in range(int(r.integers(2, 7))):
        vis = int(r.integers(1, 400))
        seqs.append((int(r.integers(0, 10)), vis, base.n_query + int(r.integers(0, 20)),
                     int(r.integers(0, vis + 1))))
    return base, seqs


def test_random_ragged_batches():
    """Random per-sequence lengths, spans and budgets through both ragged entry points."""
    import torch
    r = np.random.default_rng(20250523)
    for i in range(16):
        fused = i % 2 == 1
        base, seqs = _ragged_draw(r, fused)
        print("ragged", i, "fused" if fused else "qk", base, seqs, flush=True)
        if fused:
            caps, meta, inp, refs = pu.ragged_fused_case(base, seqs, seed=33000 + 53 * i)
            out = vb.llm_prune_fused_ragged(
                caps, meta, pu.to_device(inp["hidden"], caps.dtype), pu.to_device(inp["w_q"], caps.dtype),
                pu.to_device(np.ascontiguousarray(inp["w_k"].T), caps.dtype), want_scores=True)
            torch.cuda.synchronize()
            pu.check_fused_ragged(caps, meta, inp, refs, out, caps.in_place, f"ragged {i}")
        else:
            caps, meta, inp, refs = pu.ragged_llm_case(base, seqs, seed=33000 + 53 * i)
            q, k, v, h = (pu.to_device(inp[n], caps.dtype) for n in ("q", "k", "v", "hidden"))
            out = vb.llm_prune_ragged(caps, meta, q, k, v, h, want_scores=True)
            torch.cuda.synchronize()
            pu.check_llm_ragged(caps, meta, inp, refs, out, caps.in_place, f"ragged {i}")
