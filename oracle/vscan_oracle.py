"""ctypes front end of the CPU oracle (oracle/vscan_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product path.  It marshals numpy
arrays and chains the C functions in the paper's order (Sec. 4.1: score ->
local/global select -> assign -> merge; Sec. 4.2: score -> top-k -> compaction).
Its own arithmetic is limited to the two functions that write Eq. 1 and Eq. 5 out
from hidden states and projection weights (`encoder_scores_from_hidden`,
`llm_scores_from_hidden`: project, softmax, head mean, in numpy fp64), pinned
in tests/test_oracle_pins.py by closed forms and against the C functions.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vscan_oracle.c")
_LIB = os.path.join(_HERE, "libvscan_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over independent items)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.vso_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(_load().vso_threads())


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _f64p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with status {rc}")


def default_scale(head_dim: int, scale: float = 0.0) -> float:
    return float(scale) if scale > 0 else 1.0 / math.sqrt(head_dim)


def encoder_scores(q, k, has_cls: int, mode: int, domain: int = 0, scale: float = 0.0):
    """q, k: [B,C,H,S,dh] -> scores [B,C,N] fp64 (Eq. 1-2 / mean attention received)."""
    q, qp = _f32(q)
    k, kp = _f32(k)
    B, C, H, S, dh = q.shape
    assert k.shape == q.shape
    N = S - has_cls
    out = np.empty((B, C, N), dtype=np.float64)
    rc = _load().vso_encoder_scores(qp, kp, B, C, H, S, dh, int(has_cls), int(mode), int(domain),
                                    ctypes.c_double(default_scale(dh, scale)), _f64p(out))
    _check(rc, "encoder_scores")
    return out


def select(s_local, s_global, gh, gw, wr, wc, kl, kg):
    """scores [B,C,N] -> kept [B, C*(kl+kg)] int32, ascending per image (Eq. 2-3)."""
    s_local = np.ascontiguousarray(s_local, dtype=np.float64)
    s_global = np.ascontiguousarray(s_global, dtype=np.float64)
    B, C, N = s_global.shape
    assert N == gh * gw and s_local.shape == s_global.shape
    kept = np.empty((B, C * (kl + kg)), dtype=np.int32)
    rc = _load().vso_select(_f64p(s_local), _f64p(s_global), B, C, gh, gw, wr, wc, kl, kg,
                            kept.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    _check(rc, "select")
    return kept


def assign(x, kept):
    """x [B,T,D], kept [B,K] -> slot of every token [B,T] (highest cosine, first on ties)."""
    x, xp = _f32(x)
    kept, kp = _i32(kept)
    B, T, D = x.shape
    K = kept.shape[1]
    out = np.empty((B, T), dtype=np.int32)
    rc = _load().vso_assign(xp, kp, B, T, D, K, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    _check(rc, "assign")
    return out


def merge(x, kept, assign_):
    """Eq. 4 under a given assignment -> (merged [B,K,D] fp64, counts [B,K])."""
    x, xp = _f32(x)
    kept, kp = _i32(kept)
    assign_, ap = _i32(assign_)
    B, T, D = x.shape
    K = kept.shape[1]
    merged = np.empty((B, K, D), dtype=np.float64)
    counts = np.empty((B, K), dtype=np.int32)
    rc = _load().vso_merge(xp, kp, ap, B, T, D, K, _f64p(merged),
                           counts.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    _check(rc, "merge")
    return merged, counts


def cos_pairs(x, u, s):
    """Cosine similarity of rows u[i], s[i] of x viewed as [rows, D] (flat row indices)."""
    x, xp = _f32(x)
    D = x.shape[-1]
    u = np.ascontiguousarray(u, dtype=np.int64)
    s = np.ascontiguousarray(s, dtype=np.int64)
    out = np.empty(u.shape, dtype=np.float64)
    rc = _load().vso_cos_pairs(xp, D, ctypes.c_int64(u.size),
                               u.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                               s.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), _f64p(out))
    _check(rc, "cos_pairs")
    return out


def llm_scores(q, k, vis_start, V, domain: int = 0, scale: float = 0.0):
    """q [B,Hq,Tq,dh], k [B,Hkv,S,dh] -> scores [B,V] fp64 (Eq. 5, head/query mean)."""
    q, qp = _f32(q)
    k, kp = _f32(k)
    B, Hq, Tq, dh = q.shape
    _, Hkv, S, _ = k.shape
    out = np.empty((B, V), dtype=np.float64)
    rc = _load().vso_llm_scores(qp, kp, B, Hq, Hkv, Tq, S, dh, vis_start, V, int(domain),
                                ctypes.c_double(default_scale(dh, scale)), _f64p(out))
    _check(rc, "llm_scores")
    return out


def topk(scores, keep):
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    B, V = scores.shape
    kept = np.empty((B, keep), dtype=np.int32)
    rc = _load().vso_topk(_f64p(scores), B, V, keep,
                          kept.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    _check(rc, "topk")
    return kept


def compact(t, kept, vis_start, V):
    """t [B,G,S,W] (or [B,S,W]) -> [B,G,S_out,W]: prefix ++ kept visual ++ tail rows."""
    t, tp = _f32(t)
    squeeze = t.ndim == 3
    if squeeze:
        t = t[:, None]
    kept, kp = _i32(kept)
    B, G, S, W = t.shape
    keep = kept.shape[1]
    out = np.empty((B, G, S - V + keep, W), dtype=np.float32)
    rc = _load().vso_compact(tp, kp, B, G, S, W, vis_start, V, keep,
                             out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    _check(rc, "compact")
    return out[:, 0] if squeeze else out


def encoder_reduce(shape, q, k, x, q_local=None, k_local=None) -> Dict[str, np.ndarray]:
    """Sec. 4.1 end to end for an `EncoderShape`-like object (duck-typed)."""
    s_global = encoder_scores(q, k, shape.has_cls, shape.score_mode, shape.softmax_domain,
                              shape.scale)
    if q_local is not None:
        s_local = encoder_scores(q_local, k_local, shape.has_cls, shape.score_mode,
                                 shape.softmax_domain, shape.scale)
    else:
        s_local = s_global
    kept = select(s_local, s_global, shape.grid_h, shape.grid_w, shape.win_rows, shape.win_cols,
                  shape.keep_local, shape.keep_global)
    a = assign(x, kept)
    merged, counts = merge(x, kept, a)
    return {"scores": s_global.reshape(s_global.shape[0], -1),
            "scores_local": s_local.reshape(s_local.shape[0], -1),
            "kept": kept, "assign": a, "merged": merged, "counts": counts}


def llm_prune(shape, q, k, v, hidden) -> Dict[str, np.ndarray]:
    """Sec. 4.2 end to end for an `LlmShape`-like object (duck-typed)."""
    s = llm_scores(q, k, shape.vis_start, shape.vis_len, shape.softmax_domain, shape.scale)
    kept = topk(s, shape.keep)
    return {"scores": s, "kept": kept,
            "k": compact(k, kept, shape.vis_start, shape.vis_len),
            "v": compact(v, kept, shape.vis_start, shape.vis_len),
            "hidden": compact(hidden, kept, shape.vis_start, shape.vis_len)}


def llm_scores_from_hidden(hidden, w_q, w_k, vis_start, V, n_query, q_heads, kv_heads, head_dim,
                           domain: int = 0, scale: float = 0.0):
    """Eq. 5 written out from the hidden states (Sec. 4.2): with the layer's projection weights
    w_q [Hq*dh, Dh], w_k [Hkv*dh, Dh] (rows = output features),
        Q = x_last W_Q^h,  K = x W_K^h,  S^h = softmax(Q K^T * scale)   per head h,
    then the mean over query heads (and over the last n_query positions, an extension of the
    paper's single last token).  hidden [B,S,Dh] -> scores [B,V] fp64.  Plain numpy in fp64.
    domain 0: the softmax runs over the visual keys only, as the equation is written;
    domain 1: over the causal row of each query - query t of the last n_query positions sees
    keys 0 .. S - n_query + t - and the visual columns are taken (the two readings of
    llm_scores)."""
    x = np.asarray(hidden, dtype=np.float64)
    wq = np.asarray(w_q, dtype=np.float64)
    wk = np.asarray(w_k, dtype=np.float64)
    B, S, Dh = x.shape
    sc = default_scale(head_dim, scale)
    group = q_heads // kv_heads
    q = (x[:, S - n_query:, :] @ wq.T).reshape(B, n_query, q_heads, head_dim)
    k = (x @ wk.T).reshape(B, S, kv_heads, head_dim)
    out = np.zeros((B, V), dtype=np.float64)
    for b in range(B):
        for h in range(q_heads):
            for t in range(n_query):
                k0, nk = (0, S - n_query + t + 1) if domain else (vis_start, V)
                logit = k[b, k0:k0 + nk, h // group, :] @ q[b, t, h] * sc
                e = np.exp(logit - logit.max())
                out[b] += (e / e.sum())[vis_start - k0:vis_start - k0 + V]
    return out / (q_heads * n_query)


def llm_prune_fused(shape, hidden, w_q, w_k) -> Dict[str, np.ndarray]:
    """Stage 2 from the hidden states alone: Eq. 5 scores, top-keep, compaction of the hidden
    states (K and V of the layer do not exist yet and are computed on what is left)."""
    s = llm_scores_from_hidden(hidden, w_q, w_k, shape.vis_start, shape.vis_len, shape.n_query,
                               shape.q_heads, shape.kv_heads, shape.head_dim,
                               shape.softmax_domain, shape.scale)
    kept = topk(s, shape.keep)
    return {"scores": s, "kept": kept,
            "hidden": compact(hidden, kept, shape.vis_start, shape.vis_len)}


def encoder_scores_from_hidden(hidden, w_q, w_k, heads, head_dim, domain: int = 0,
                               scale: float = 0.0):
    """Eq. 1-2 written out from the rows the attention layer sees (Sec. 4.1 "Global Scan"):
    hidden [B,C,S,D] with the [CLS] row first, w_q, w_k [H*dh, D] (rows = output features),
        Q = x_CLS W_Q^h,  K = x W_K^h,  S^h = softmax(Q K^T * scale),  S_avg = mean over heads.
    Returns the [CLS] row's attention to the N = S-1 patch tokens, [B,C,N] fp64.  domain 0: the
    softmax runs over the patch keys only; domain 1: over all S keys ([CLS] included) and the
    patch columns are taken (the two readings of `encoder_scores`).  Plain numpy in fp64."""
    x = np.asarray(hidden, dtype=np.float64)
    wq = np.asarray(w_q, dtype=np.float64)
    wk = np.asarray(w_k, dtype=np.float64)
    B, C, S, D = x.shape
    sc = default_scale(head_dim, scale)
    k0 = 0 if domain else 1
    q = (x[:, :, 0, :] @ wq.T).reshape(B, C, heads, head_dim)
    k = (x[:, :, k0:, :] @ wk.T).reshape(B, C, S - k0, heads, head_dim)
    out = np.zeros((B, C, S - 1), dtype=np.float64)
    for b in range(B):
        for c in range(C):
            for h in range(heads):
                logit = k[b, c, :, h, :] @ q[b, c, h] * sc
                e = np.exp(logit - logit.max())
                out[b, c] += (e / e.sum())[1 - k0:]
    return out / heads


def encoder_mean_scores_from_hidden(hidden, w_q, w_k, heads, head_dim, has_cls: int,
                                    domain: int = 0, scale: float = 0.0):
    """The encoder without a usable [CLS] row (last sentence of Sec. 4.1 "Global Scan"), written
    out from the rows the attention layer sees: hidden [B,C,S,D] (S = N + has_cls, the [CLS] row
    first where there is one), w_q, w_k [H*dh, D],
        Q = x W_Q^h,  K = x W_K^h,  A^h = row-softmax(Q K^T * scale) for the N patch queries,
        score_j = mean over heads and over the N queries of A^h_ij  (diagonal included).
    domain 0: the softmax runs over the patch keys; domain 1: over all S keys, and the [CLS]
    column is dropped afterwards.  Returns [B,C,N] fp64.  Plain numpy in fp64."""
    x = np.asarray(hidden, dtype=np.float64)
    wq = np.asarray(w_q, dtype=np.float64)
    wk = np.asarray(w_k, dtype=np.float64)
    B, C, S, D = x.shape
    N = S - has_cls
    sc = default_scale(head_dim, scale)
    k0 = 0 if domain else has_cls
    out = np.zeros((B, C, N), dtype=np.float64)
    for b in range(B):
        for c in range(C):
            q = (x[b, c, has_cls:, :] @ wq.T).reshape(N, heads, head_dim)
            k = (x[b, c, k0:, :] @ wk.T).reshape(S - k0, heads, head_dim)
            for h in range(heads):
                logit = q[:, h, :] @ k[:, h, :].T * sc              # [N queries, keys]
                e = np.exp(logit - logit.max(axis=1, keepdims=True))
                a = e / e.sum(axis=1, keepdims=True)
                out[b, c] += a[:, has_cls - k0:].sum(axis=0)
    return out / (heads * N)


def encoder_reduce_fused(shape, hidden, w_q, w_k, x, hidden_local=None, w_q_local=None,
                         w_k_local=None) -> Dict[str, np.ndarray]:
    """Sec. 4.1 end to end with the scores taken from hidden states and projection weights
    ([CLS] row or mean attention received, as the shape says); the optional second triple is the
    shallow layer of the local scan."""
    def scores(h, wq, wk):
        if shape.score_mode == 1:
            return encoder_mean_scores_from_hidden(h, wq, wk, shape.heads, shape.head_dim,
                                                   shape.has_cls, shape.softmax_domain, shape.scale)
        return encoder_scores_from_hidden(h, wq, wk, shape.heads, shape.head_dim,
                                          shape.softmax_domain, shape.scale)
    s_global = scores(hidden, w_q, w_k)
    if hidden_local is not None:
        s_local = scores(hidden_local, w_q_local, w_k_local)
    else:
        s_local = s_global
    kept = select(s_local, s_global, shape.grid_h, shape.grid_w, shape.win_rows, shape.win_cols,
                  shape.keep_local, shape.keep_global)
    a = assign(x, kept)
    merged, counts = merge(x, kept, a)
    return {"scores": s_global.reshape(s_global.shape[0], -1),
            "scores_local": s_local.reshape(s_local.shape[0], -1),
            "kept": kept, "assign": a, "merged": merged, "counts": counts}
