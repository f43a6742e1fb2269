"""Seeded synthetic inputs shaped like the paper's LVLM workloads.

This module only draws random tensors and names shapes.  It holds none of the
method's arithmetic (no softmax, no selection, no similarity, no merging): the
HIP path and the CPU oracle both consume what it produces and share nothing
else.

The inputs stand in for the visual-encoder and mid-LLM-layer tensors of the
models the paper evaluates (Sec. 5.1, "Models": LLaVA-1.5 with 576 visual
tokens, LLaVA-NeXT with up to 2880, Qwen-2.5-VL with up to 16384).  No model
weight and no benchmark item is used.

Recipe
------
Encoder stage, per image and per segment (crop):
  * 48 cluster centres c_m ~ N(0, 1)^D, one set per image;
  * every patch token draws a cluster id uniformly, x = c_m + N(0, 0.1^2)^D;
  * 4 patch tokens per segment (distinct random positions) are scaled by 3;
  * where a [CLS] row exists its feature is the mean of the segment's patch
    features plus N(0, 0.1^2)^D noise;
  * W_Q, W_K in R^{D x (H*dh)} with N(0, 1/64) entries (variance 1/64), one pair
    per workload; q = gain * x W_Q, k = x W_K for every row incl. [CLS].
LLM stage, per sequence: q, K, V and hidden states are iid N(0, 1); 4 visual
keys per (sequence, kv head) are nudged towards the mean query direction so a
non-trivial top set exists.

Everything is generated in fp64 with numpy's PCG64, cast to fp32, and for
bf16 workloads rounded (nearest-even) to bf16-representable fp32 values, so
both consumers read identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

BASE_SEED = 20250522

F32 = "f32"
BF16 = "bf16"


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable value (ties to even).

    The result is still an fp32 array; its low 16 mantissa bits are zero."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    u = ((u + bias) & 0xFFFF0000).astype(np.uint32)
    return u.view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of bf16-representable fp32 values, as int16 (for upload)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).view(np.int16).reshape(a.shape)


@dataclass(frozen=True)
class EncoderShape:
    """Shape of one `vscan_encoder_reduce` call (Sec. 4.1)."""
    dtype: str
    batch: int
    n_segments: int
    grid_h: int
    grid_w: int
    has_cls: int
    score_mode: int          # 0: [CLS] row, 1: mean attention received
    heads: int
    head_dim: int
    feat_dim: int
    win_rows: int
    win_cols: int
    keep_global: int         # per segment
    keep_local: int          # per segment
    softmax_domain: int = 0  # 0: visual keys only, 1: all keys
    scale: float = 0.0       # <= 0: 1/sqrt(head_dim)

    @property
    def n_tokens(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def rows(self) -> int:
        return self.n_tokens + (1 if self.has_cls else 0)

    @property
    def keep(self) -> int:
        return self.n_segments * (self.keep_global + self.keep_local)

    @property
    def tokens_per_image(self) -> int:
        return self.n_segments * self.n_tokens


@dataclass(frozen=True)
class LlmShape:
    """Shape of one `vscan_llm_prune` call (Sec. 4.2)."""
    dtype: str
    batch: int
    prefix: int
    vis_len: int
    text: int
    n_query: int
    q_heads: int
    kv_heads: int
    head_dim: int
    hidden: int
    keep: int
    in_place: int = 0
    softmax_domain: int = 0
    scale: float = 0.0

    @property
    def seq_len(self) -> int:
        return self.prefix + self.vis_len + self.text

    @property
    def vis_start(self) -> int:
        return self.prefix

    @property
    def seq_out(self) -> int:
        return self.seq_len - self.vis_len + self.keep


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    encoder: Optional[EncoderShape]
    llm: Optional[LlmShape]
    note: str = ""


def _enc_llava(dtype, batch, crops, keep_total_per_seg, win, grid=24):
    half = keep_total_per_seg // 2
    return EncoderShape(dtype=dtype, batch=batch, n_segments=crops, grid_h=grid, grid_w=grid,
                        has_cls=1, score_mode=0, heads=16, head_dim=64, feat_dim=1024,
                        win_rows=win, win_cols=win, keep_global=keep_total_per_seg - half,
                        keep_local=half)


def _llm_llama(dtype, batch, prefix, vis, text, keep, n_query=1, in_place=0):
    return LlmShape(dtype=dtype, batch=batch, prefix=prefix, vis_len=vis, text=text,
                    n_query=n_query, q_heads=32, kv_heads=32, head_dim=128, hidden=4096,
                    keep=keep, in_place=in_place)


def config(index: int, sweep: Optional[int] = None, batch: Optional[int] = None) -> Workload:
    """The benchmark configurations (1-based index; 6 is a video shape: 8 frames of 16x16
    patches, 2048 visual tokens, at the 25 % average budget of the paper's video table).

    `sweep` picks the keep budget where a configuration sweeps one: the encoder
    keep {192,128,64} for 2 and the LLM keep {720,288,144} for 5."""
    seed = BASE_SEED + index
    if index == 1:
        enc = _enc_llava(F32, 1, 1, 64, 2)
        llm = _llm_llama(F32, 1, 35, 64, 40, 32)
        w = Workload("cfg1-clip-tiny-f32", seed, enc, llm)
    elif index == 2:
        k = 192 if sweep is None else sweep
        assert k in (192, 128, 64)
        enc = _enc_llava(BF16, 16, 1, k, 4)
        llm = _llm_llama(BF16, 16, 35, k, 64, k // 2)
        w = Workload(f"cfg2-llava15-b16-keep{k}", seed, enc, llm)
    elif index == 3:
        enc = _enc_llava(BF16, 8, 5, 64, 4)
        llm = _llm_llama(BF16, 8, 35, 320, 128, 160)
        w = Workload("cfg3-llavanext-b8", seed, enc, llm)
    elif index == 4:
        enc = EncoderShape(dtype=BF16, batch=1, n_segments=1, grid_h=128, grid_w=128, has_cls=0,
                           score_mode=1, heads=16, head_dim=80, feat_dim=1280, win_rows=8,
                           win_cols=8, keep_global=2048, keep_local=2048)
        llm = LlmShape(dtype=BF16, batch=1, prefix=0, vis_len=4096, text=256, n_query=1,
                       q_heads=28, kv_heads=4, head_dim=128, hidden=3584, keep=2048)
        w = Workload("cfg4-qwen25vl-16k", seed, enc, llm)
    elif index == 5:
        k = 720 if sweep is None else sweep
        assert k in (720, 288, 144)
        llm = _llm_llama(BF16, 32, 35, 2880, 512, k, n_query=8, in_place=1)
        w = Workload(f"cfg5-llm-stress-keep{k}", seed, None, llm)
    elif index == 6:
        # 25 % average retention at R2 = 33.3 %, middle-layer pruning: R1 = 37.5 %, i.e. 96 of
        # 256 tokens per frame (768 per video) before the LLM and 256 after (average 512 of 2048)
        enc = _enc_llava(BF16, 4, 8, 96, 4, grid=16)
        llm = _llm_llama(BF16, 4, 35, 768, 64, 256)
        w = Workload("cfg6-video-8frames-b4", seed, enc, llm)
    else:
        raise ValueError("config index must be 1..6")
    if batch is not None:
        w = replace(w, encoder=None if w.encoder is None else replace(w.encoder, batch=batch),
                    llm=None if w.llm is None else replace(w.llm, batch=batch))
    return w


def _finish(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return round_to_bf16(a) if dtype == BF16 else a


def _rng(seed: int, *stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, *stream])))


N_CENTRES = 48
N_BOOST = 4


def encoder_projections(shape: EncoderShape, seed: int):
    """The workload-wide random projections W_Q, W_K (fp64)."""
    r = _rng(seed, 1_000_003)
    hd = shape.heads * shape.head_dim
    wq = r.normal(0.0, 0.125, size=(shape.feat_dim, hd))
    wk = r.normal(0.0, 0.125, size=(shape.feat_dim, hd))
    return wq, wk


def _encoder_rows(shape: EncoderShape, seed: int, b: int, stream: int):
    """Features of image `b` in fp64: x [C,N,D] (patch tokens) and rows [C,S,D] (the rows the
    attention layer sees: [CLS] first where there is one)."""
    C, N, S, D = shape.n_segments, shape.n_tokens, shape.rows, shape.feat_dim
    r = _rng(seed, b, 0)
    centres = r.normal(0.0, 1.0, size=(N_CENTRES, D))
    x = np.empty((C, N, D))
    rows = np.empty((C, S, D))
    for c in range(C):
        ids = r.integers(0, N_CENTRES, size=N)
        xc = centres[ids] + r.normal(0.0, 0.1, size=(N, D))
        boost = r.choice(N, size=min(N_BOOST, N), replace=False)
        xc[boost] *= 3.0
        x[c] = xc
        if shape.has_cls:
            rows[c, 0] = xc.mean(axis=0) + r.normal(0.0, 0.1, size=D)
            rows[c, 1:] = xc
        else:
            rows[c] = xc
    if stream != 0:
        # a second, independent view of the same image for the shallow layer:
        # the same features perturbed, so local and global rankings differ
        r2 = _rng(seed, b, stream)
        rows = rows + r2.normal(0.0, 0.5, size=rows.shape)
    return x, rows


def encoder_item(shape: EncoderShape, seed: int, b: int, logit_gain: float = 1.0,
                 proj=None, stream: int = 0) -> Dict[str, np.ndarray]:
    """Inputs of image `b`: q, k [C,H,S,dh] and x [C*N,D] as fp32 arrays.

    `stream` selects an independent draw of the features behind q/k only (used
    for the shallow-layer pair of the local scan); x always comes from stream 0."""
    C, N, S = shape.n_segments, shape.n_tokens, shape.rows
    H, dh, D = shape.heads, shape.head_dim, shape.feat_dim
    wq, wk = proj if proj is not None else encoder_projections(shape, seed)
    x, rows = _encoder_rows(shape, seed, b, stream)
    q = (rows.reshape(C * S, D) @ wq) * logit_gain
    k = rows.reshape(C * S, D) @ wk
    q = q.reshape(C, S, H, dh).transpose(0, 2, 1, 3)
    k = k.reshape(C, S, H, dh).transpose(0, 2, 1, 3)
    return {
        "q": _finish(q, shape.dtype),
        "k": _finish(k, shape.dtype),
        "x": _finish(x.reshape(C * N, D), shape.dtype),
    }


def encoder_hidden_inputs(shape: EncoderShape, seed: int, logit_gain: float = 1.0,
                          stream: int = 0) -> Dict[str, np.ndarray]:
    """Whole batch for the form of stage 1 that scores from the layer's input rows and its
    projection weights: hidden [B,C,S,D] (the rows behind q and k of `encoder_inputs`, rounded
    to the workload's dtype), x [B,C*N,D], w_q and w_k [H*dh, D] (rows = output features; the
    logit gain is folded into w_q)."""
    wq, wk = encoder_projections(shape, seed)
    hidden, xs = [], []
    for b in range(shape.batch):
        x, rows = _encoder_rows(shape, seed, b, stream)
        hidden.append(rows)
        xs.append(x.reshape(shape.n_segments * shape.n_tokens, shape.feat_dim))
    return {"hidden": _finish(np.stack(hidden), shape.dtype), "x": _finish(np.stack(xs), shape.dtype),
            "w_q": _finish((wq * logit_gain).T, shape.dtype), "w_k": _finish(wk.T, shape.dtype)}


def encoder_inputs(shape: EncoderShape, seed: int, logit_gain: float = 1.0,
                   stream: int = 0) -> Dict[str, np.ndarray]:
    """Whole batch: q, k [B,C,H,S,dh], x [B,C*N,D]."""
    proj = encoder_projections(shape, seed)
    items = [encoder_item(shape, seed, b, logit_gain, proj, stream) for b in range(shape.batch)]
    return {key: np.stack([it[key] for it in items]) for key in ("q", "k", "x")}


N_NUDGE = 4


def llm_item(shape: LlmShape, seed: int, b: int) -> Dict[str, np.ndarray]:
    """Inputs of sequence `b`: q [Hq,Tq,dh], k, v [Hkv,S,dh], hidden [S,Dh] (fp32)."""
    r = _rng(seed, b, 7)
    Hq, Hkv, dh, S = shape.q_heads, shape.kv_heads, shape.head_dim, shape.seq_len
    q = r.standard_normal(size=(Hq, shape.n_query, dh), dtype=np.float32)
    k = r.standard_normal(size=(Hkv, S, dh), dtype=np.float32)
    v = r.standard_normal(size=(Hkv, S, dh), dtype=np.float32)
    hidden = r.standard_normal(size=(S, shape.hidden), dtype=np.float32)
    group = Hq // Hkv
    n_nudge = min(N_NUDGE, shape.vis_len)
    pos = r.choice(shape.vis_len, size=n_nudge, replace=False) + shape.vis_start
    for g in range(Hkv):
        direction = q[g * group:(g + 1) * group].mean(axis=(0, 1))
        k[g, pos] += np.float32(0.5) * direction
    return {"q": _finish(q, shape.dtype), "k": _finish(k, shape.dtype),
            "v": _finish(v, shape.dtype), "hidden": _finish(hidden, shape.dtype)}


def llm_weights(shape: LlmShape, seed: int) -> Dict[str, np.ndarray]:
    """Projection weights of the pruning layer for the fused form of stage 2: w_q [Hq*dh, Dh],
    w_k [Hkv*dh, Dh], rows = output features, entries N(0, 1/Dh) so that projected queries and
    keys of N(0,1) hidden states have unit-variance components."""
    r = _rng(seed, 2_000_003)
    sd = 1.0 / np.sqrt(shape.hidden)
    wq = r.normal(0.0, sd, size=(shape.q_heads * shape.head_dim, shape.hidden)).astype(np.float32)
    wk = r.normal(0.0, sd, size=(shape.kv_heads * shape.head_dim, shape.hidden)).astype(np.float32)
    return {"w_q": _finish(wq, shape.dtype), "w_k": _finish(wk, shape.dtype)}


def llm_inputs(shape: LlmShape, seed: int) -> Dict[str, np.ndarray]:
    """Whole batch: q [B,Hq,Tq,dh], k, v [B,Hkv,S,dh], hidden [B,S,Dh]."""
    items = [llm_item(shape, seed, b) for b in range(shape.batch)]
    return {key: np.stack([it[key] for it in items]) for key in ("q", "k", "v", "hidden")}
