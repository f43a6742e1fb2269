"""Thin ctypes binding of libvscan.so (include/vscan.h).

Argument marshalling only: every step of the reduction runs in the HIP kernels
behind the C ABI.  torch is used for device memory and the current stream.
There is no fallback: if the library is missing the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libvscan.so")
_lib = None

VSCAN_F32, VSCAN_BF16 = 0, 1
VSCAN_SCORE_CLS_ROW, VSCAN_SCORE_MEAN_RECEIVED = 0, 1
VSCAN_KEYS_VISUAL_ONLY, VSCAN_KEYS_ALL = 0, 1
(VSCAN_OK, VSCAN_ERR_NULL, VSCAN_ERR_SHAPE, VSCAN_ERR_BUDGET, VSCAN_ERR_DTYPE, VSCAN_ERR_ALIGN,
 VSCAN_ERR_WORKSPACE, VSCAN_ERR_HIP, VSCAN_ERR_VERSION, VSCAN_ERR_UNSUPPORTED) = (
    0, -1, -2, -3, -4, -5, -6, -7, -8, -9)

EXPORTS = ("vscan_encoder_workspace_size", "vscan_encoder_reduce", "vscan_llm_workspace_size",
           "vscan_llm_prune", "vscan_profile_enable", "vscan_profile_read", "vscan_status_string",
           "vscan_version", "vscan_budget", "vscan_budget_solve_r1", "vscan_flops",
           "vscan_llm_prune_ragged", "vscan_llm_fused_workspace_size", "vscan_llm_prune_fused",
           "vscan_encoder_fused_workspace_size", "vscan_encoder_reduce_fused",
           "vscan_llm_prune_fused_ragged", "vscan_llm_prune_static")
STATIC_SCRATCH_BYTES = 16 << 20


class EncoderDesc(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("batch", ctypes.c_int32), ("n_segments", ctypes.c_int32),
                ("grid_h", ctypes.c_int32), ("grid_w", ctypes.c_int32),
                ("has_cls", ctypes.c_int32), ("score_mode", ctypes.c_int32),
                ("softmax_domain", ctypes.c_int32), ("heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("feat_dim", ctypes.c_int32),
                ("win_rows", ctypes.c_int32), ("win_cols", ctypes.c_int32),
                ("keep_global", ctypes.c_int32), ("keep_local", ctypes.c_int32),
                ("scale", ctypes.c_float)]


class LlmDesc(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("batch", ctypes.c_int32), ("seq_len", ctypes.c_int32),
                ("vis_start", ctypes.c_int32), ("vis_len", ctypes.c_int32),
                ("n_query", ctypes.c_int32), ("q_heads", ctypes.c_int32),
                ("kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("hidden", ctypes.c_int32), ("keep", ctypes.c_int32),
                ("softmax_domain", ctypes.c_int32), ("in_place", ctypes.c_int32),
                ("scale", ctypes.c_float)]


class KernelTime(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 32), ("launches", ctypes.c_int32),
                ("total_ms", ctypes.c_float)]


class VscanError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib():
    """Load libvscan.so; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2505_22654_amd.build` (no CPU fallback exists)")
        # torch first: its wheel carries its own HIP runtime, found through the file name
        # libamdhip64.so, while this library asks for the soname libamdhip64.so.7.  Loaded in
        # that order the second request is satisfied by the runtime already in the process;
        # the other way round the process ends up with two runtimes (streams and device
        # pointers of one mean nothing to the other).
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32p, f32p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
        L.vscan_encoder_workspace_size.argtypes = [ctypes.POINTER(EncoderDesc), ctypes.c_int,
                                                   ctypes.POINTER(ctypes.c_size_t)]
        L.vscan_encoder_workspace_size.restype = ctypes.c_int
        L.vscan_encoder_reduce.argtypes = [ctypes.POINTER(EncoderDesc), vp, vp, vp, vp, vp, i32p,
                                           vp, i32p, f32p, vp, ctypes.c_size_t, vp]
        L.vscan_encoder_reduce.restype = ctypes.c_int
        L.vscan_llm_workspace_size.argtypes = [ctypes.POINTER(LlmDesc),
                                               ctypes.POINTER(ctypes.c_size_t)]
        L.vscan_llm_workspace_size.restype = ctypes.c_int
        L.vscan_llm_prune.argtypes = [ctypes.POINTER(LlmDesc), vp, vp, vp, vp, i32p, vp, vp, vp,
                                      f32p, vp, ctypes.c_size_t, vp]
        L.vscan_llm_prune.restype = ctypes.c_int
        L.vscan_llm_prune_static.argtypes = [ctypes.POINTER(LlmDesc), vp, vp, vp, vp, i32p, vp, vp,
                                             vp, f32p, vp]
        L.vscan_llm_prune_static.restype = ctypes.c_int
        L.vscan_llm_prune_ragged.argtypes = [ctypes.POINTER(LlmDesc), vp, vp, vp, vp, vp, vp, i32p,
                                             vp, vp, vp, f32p, vp, ctypes.c_size_t, vp]
        L.vscan_llm_prune_ragged.restype = ctypes.c_int
        L.vscan_llm_fused_workspace_size.argtypes = [ctypes.POINTER(LlmDesc),
                                                     ctypes.POINTER(ctypes.c_size_t)]
        L.vscan_llm_fused_workspace_size.restype = ctypes.c_int
        L.vscan_llm_prune_fused.argtypes = [ctypes.POINTER(LlmDesc), vp, vp, vp, i32p, vp, f32p, vp,
                                            ctypes.c_size_t, vp]
        L.vscan_llm_prune_fused.restype = ctypes.c_int
        L.vscan_encoder_fused_workspace_size.argtypes = [ctypes.POINTER(EncoderDesc), ctypes.c_int,
                                                         ctypes.POINTER(ctypes.c_size_t)]
        L.vscan_encoder_fused_workspace_size.restype = ctypes.c_int
        L.vscan_encoder_reduce_fused.argtypes = [ctypes.POINTER(EncoderDesc), vp, vp, vp, vp, vp, vp,
                                                 vp, i32p, vp, i32p, f32p, vp, ctypes.c_size_t, vp]
        L.vscan_encoder_reduce_fused.restype = ctypes.c_int
        L.vscan_llm_prune_fused_ragged.argtypes = [ctypes.POINTER(LlmDesc), vp, vp, vp, vp, vp, i32p,
                                                   vp, f32p, vp, ctypes.c_size_t, vp]
        L.vscan_llm_prune_fused_ragged.restype = ctypes.c_int
        L.vscan_profile_enable.argtypes = [ctypes.c_int]
        L.vscan_profile_enable.restype = ctypes.c_int
        L.vscan_profile_read.argtypes = [ctypes.POINTER(KernelTime), ctypes.c_int,
                                         ctypes.POINTER(ctypes.c_int)]
        L.vscan_profile_read.restype = ctypes.c_int
        L.vscan_status_string.argtypes = [ctypes.c_int]
        L.vscan_status_string.restype = ctypes.c_char_p
        L.vscan_version.restype = ctypes.c_uint32
        dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
        L.vscan_budget.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                   ctypes.c_double, ip, ip, dp]
        L.vscan_budget.restype = ctypes.c_int
        L.vscan_budget_solve_r1.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                            ctypes.c_double, dp]
        L.vscan_budget_solve_r1.restype = ctypes.c_int
        L.vscan_flops.argtypes = [ip, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, dp]
        L.vscan_flops.restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().vscan_status_string(int(status)).decode()


def version() -> int:
    return int(lib().vscan_version())


def profile_enable(on: bool) -> None:
    """Switch per-kernel event timing inside the library on or off."""
    lib().vscan_profile_enable(int(on))


def profile_read() -> Dict[str, Dict[str, float]]:
    """{kernel name: {"launches": n, "total_ms": t}} since the last read."""
    buf = (KernelTime * 32)()
    n = ctypes.c_int(0)
    rc = lib().vscan_profile_read(buf, 32, ctypes.byref(n))
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_profile_read")
    return {buf[i].name.decode(): {"launches": int(buf[i].launches),
                                   "total_ms": float(buf[i].total_ms)} for i in range(n.value)}


def budget(n_visual: int, n_layers: int, prune_layer: int, r1: float, r2: float):
    """(keep_encoder, keep_llm, average tokens over the LLM layers) for retention rates r1, r2."""
    n1, n2, avg = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_double(0.0)
    rc = lib().vscan_budget(n_visual, n_layers, prune_layer, r1, r2, ctypes.byref(n1),
                            ctypes.byref(n2), ctypes.byref(avg))
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_budget")
    return int(n1.value), int(n2.value), float(avg.value)


def budget_solve_r1(n_layers: int, prune_layer: int, avg_rate: float, r2: float) -> float:
    """Stage-1 retention rate that gives the layer-averaged retention `avg_rate` at fixed r2."""
    r1 = ctypes.c_double(0.0)
    rc = lib().vscan_budget_solve_r1(n_layers, prune_layer, avg_rate, r2, ctypes.byref(r1))
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_budget_solve_r1")
    return float(r1.value)


def flops(n_per_layer, d: int, m: int) -> float:
    """Eq. 6 for a per-layer list of visual token counts."""
    arr = (ctypes.c_int32 * max(len(n_per_layer), 1))(*[int(n) for n in n_per_layer])
    out = ctypes.c_double(0.0)
    rc = lib().vscan_flops(arr, len(n_per_layer), d, m, ctypes.byref(out))
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_flops")
    return float(out.value)


def llm_prune_ragged(shape, meta, q, k, v, hidden, want_scores: bool = False) -> Dict[str, object]:
    """vscan_llm_prune_ragged.  `shape` carries the shared fields and the capacities (seq_len,
    vis_len, keep); `meta` is a list of (seq_len, vis_start, vis_len, keep) per sequence.
    Out-of-place results are tensors shaped like the inputs (rows past a sequence's result are
    zero-filled here so that they are defined); `out_len` lists the result lengths."""
    import torch
    desc = llm_desc(shape)
    need = llm_workspace_size(desc)
    dev = q.device
    B = shape.batch
    assert len(meta) == B
    host = (ctypes.c_int32 * (4 * max(B, 1)))(*[int(x) for m in meta for x in m])
    meta_dev = torch.tensor([list(map(int, m)) for m in meta], dtype=torch.int32,
                            device=dev).reshape(B, 4).contiguous()
    workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    out = {"kept_idx": torch.empty((B, shape.keep), dtype=torch.int32, device=dev)}
    if want_scores:
        out["scores"] = torch.zeros((B, shape.vis_len), dtype=torch.float32, device=dev)
    if shape.in_place:
        ko = vo = ho = None
    else:
        ko, vo, ho = torch.zeros_like(k), torch.zeros_like(v), torch.zeros_like(hidden)
    rc = lib().vscan_llm_prune_ragged(ctypes.byref(desc), ctypes.cast(host, ctypes.c_void_p),
                                      _ptr(meta_dev), _ptr(q), _ptr(k), _ptr(v), _ptr(hidden),
                                      _ptr(out["kept_idx"]), _ptr(ko), _ptr(vo), _ptr(ho),
                                      _ptr(out.get("scores")), _ptr(workspace),
                                      workspace.numel(), _stream_handle())
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_llm_prune_ragged")
    out["k"], out["v"], out["hidden"] = (k, v, hidden) if shape.in_place else (ko, vo, ho)
    out["out_len"] = [m[0] - m[2] + m[3] for m in meta]
    out["meta_device"], out["workspace"] = meta_dev, workspace  # alive until the work has run
    return out


def _dtype_code(dtype: str) -> int:
    return {"f32": VSCAN_F32, "bf16": VSCAN_BF16}[dtype]


def encoder_desc(shape) -> EncoderDesc:
    """Descriptor from an `EncoderShape`-like object."""
    return EncoderDesc(ctypes.sizeof(EncoderDesc), _dtype_code(shape.dtype), shape.batch,
                       shape.n_segments, shape.grid_h, shape.grid_w, shape.has_cls,
                       shape.score_mode, shape.softmax_domain, shape.heads, shape.head_dim,
                       shape.feat_dim, shape.win_rows, shape.win_cols, shape.keep_global,
                       shape.keep_local, shape.scale)


def llm_desc(shape) -> LlmDesc:
    """Descriptor from an `LlmShape`-like object."""
    return LlmDesc(ctypes.sizeof(LlmDesc), _dtype_code(shape.dtype), shape.batch, shape.seq_len,
                   shape.vis_start, shape.vis_len, shape.n_query, shape.q_heads, shape.kv_heads,
                   shape.head_dim, shape.hidden, shape.keep, shape.softmax_domain, shape.in_place,
                   shape.scale)


def encoder_workspace_size(desc: EncoderDesc, with_local_pair: bool = False) -> int:
    n = ctypes.c_size_t(0)
    rc = lib().vscan_encoder_workspace_size(ctypes.byref(desc), int(with_local_pair),
                                            ctypes.byref(n))
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_encoder_workspace_size")
    return int(n.value)


def llm_workspace_size(desc: LlmDesc) -> int:
    n = ctypes.c_size_t(0)
    rc = lib().vscan_llm_workspace_size(ctypes.byref(desc), ctypes.byref(n))
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_llm_workspace_size")
    return int(n.value)


def llm_fused_workspace_size(desc: LlmDesc) -> int:
    n = ctypes.c_size_t(0)
    rc = lib().vscan_llm_fused_workspace_size(ctypes.byref(desc), ctypes.byref(n))
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_llm_fused_workspace_size")
    return int(n.value)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_handle():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _torch_dtype(dtype: str):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def encoder_reduce(shape, q, k, x, q_local=None, k_local=None, want_assign: bool = False,
                   want_scores: bool = False, workspace=None, out=None) -> Dict[str, object]:
    """vscan_encoder_reduce on CUDA tensors q, k [B,C,H,S,dh], x [B,C*N,D].

    Returns kept_idx [B,K] int32 and merged [B,K,D] (plus assign / scores on request).
    `workspace` (uint8 tensor) and `out` (dict of preallocated outputs) avoid allocation."""
    import torch
    desc = encoder_desc(shape)
    need = encoder_workspace_size(desc, q_local is not None)
    dev = q.device
    for t in (q, k, x, q_local, k_local):
        assert t is None or (t.is_cuda and t.is_contiguous() and t.dtype == _torch_dtype(shape.dtype))
    B, K, T = shape.batch, shape.keep, shape.tokens_per_image
    assert tuple(q.shape) == (B, shape.n_segments, shape.heads, shape.rows, shape.head_dim)
    assert tuple(k.shape) == tuple(q.shape) and tuple(x.shape) == (B, T, shape.feat_dim)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    out = dict(out) if out else {}
    if "kept_idx" not in out:
        out["kept_idx"] = torch.empty((B, K), dtype=torch.int32, device=dev)
    if "merged" not in out:
        out["merged"] = torch.empty((B, K, shape.feat_dim), dtype=x.dtype, device=dev)
    if want_assign and "assign" not in out:
        out["assign"] = torch.empty((B, T), dtype=torch.int32, device=dev)
    if want_scores and "scores" not in out:
        out["scores"] = torch.empty((B, T), dtype=torch.float32, device=dev)
    rc = lib().vscan_encoder_reduce(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(q_local),
                                    _ptr(k_local), _ptr(x), _ptr(out["kept_idx"]),
                                    _ptr(out["merged"]), _ptr(out.get("assign")),
                                    _ptr(out.get("scores")), _ptr(workspace), workspace.numel(),
                                    _stream_handle())
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_encoder_reduce")
    out["workspace"] = workspace
    return out


def llm_prune(shape, q, k, v, hidden, want_scores: bool = False, workspace=None,
              out=None, static_scratch: bool = False) -> Dict[str, object]:
    """vscan_llm_prune on CUDA tensors q [B,Hq,Tq,dh], k, v [B,Hkv,S,dh], hidden [B,S,Dh]
    (`static_scratch`: vscan_llm_prune_static, which takes no workspace).

    Out of place it returns k, v, hidden of length S_out; in place (shape.in_place) it
    mutates the inputs and returns views of their first S_out rows."""
    import torch
    desc = llm_desc(shape)
    need = llm_workspace_size(desc)
    dev = q.device
    for t in (q, k, v, hidden):
        assert t.is_cuda and t.is_contiguous() and t.dtype == _torch_dtype(shape.dtype)
    B, S, So = shape.batch, shape.seq_len, shape.seq_out
    assert tuple(q.shape) == (B, shape.q_heads, shape.n_query, shape.head_dim)
    assert tuple(k.shape) == (B, shape.kv_heads, S, shape.head_dim) and k.shape == v.shape
    assert tuple(hidden.shape) == (B, S, shape.hidden)
    if workspace is None and not static_scratch:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    out = dict(out) if out else {}
    if "kept_idx" not in out:
        out["kept_idx"] = torch.empty((B, shape.keep), dtype=torch.int32, device=dev)
    if want_scores and "scores" not in out:
        out["scores"] = torch.empty((B, shape.vis_len), dtype=torch.float32, device=dev)
    if shape.in_place:
        ko = vo = ho = None
    else:
        ko = out.get("k")
        vo = out.get("v")
        ho = out.get("hidden")
        if ko is None:
            ko = torch.empty((B, shape.kv_heads, So, shape.head_dim), dtype=k.dtype, device=dev)
        if vo is None:
            vo = torch.empty_like(ko)
        if ho is None:
            ho = torch.empty((B, So, shape.hidden), dtype=hidden.dtype, device=dev)
    if static_scratch:
        rc = lib().vscan_llm_prune_static(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v),
                                          _ptr(hidden), _ptr(out["kept_idx"]), _ptr(ko), _ptr(vo),
                                          _ptr(ho), _ptr(out.get("scores")), _stream_handle())
    else:
        rc = lib().vscan_llm_prune(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(hidden),
                                   _ptr(out["kept_idx"]), _ptr(ko), _ptr(vo), _ptr(ho),
                                   _ptr(out.get("scores")), _ptr(workspace), workspace.numel(),
                                   _stream_handle())
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_llm_prune_static" if static_scratch else "vscan_llm_prune")
    if shape.in_place:
        out["k"], out["v"], out["hidden"] = k[:, :, :So], v[:, :, :So], hidden[:, :So]
    else:
        out["k"], out["v"], out["hidden"] = ko, vo, ho
    out["workspace"] = workspace
    return out


def llm_prune_fused(shape, hidden, w_q, w_k_t, want_scores: bool = False, workspace=None,
                    out=None) -> Dict[str, object]:
    """vscan_llm_prune_fused on CUDA bf16 tensors hidden [B,S,Dh], w_q [Hq*dh, Dh] (rows =
    output features), w_k_t [Dh, Hkv*dh] (rows = input features).  Returns kept_idx, optional
    scores and the compacted hidden states (a view of `hidden` when shape.in_place)."""
    import torch
    desc = llm_desc(shape)
    need = llm_fused_workspace_size(desc)
    dev = hidden.device
    for t in (hidden, w_q, w_k_t):
        assert t.is_cuda and t.is_contiguous() and t.dtype == _torch_dtype(shape.dtype)
    B, S, So = shape.batch, shape.seq_len, shape.seq_out
    assert tuple(hidden.shape) == (B, S, shape.hidden)
    assert tuple(w_q.shape) == (shape.q_heads * shape.head_dim, shape.hidden)
    assert tuple(w_k_t.shape) == (shape.hidden, shape.kv_heads * shape.head_dim)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    out = dict(out) if out else {}
    if "kept_idx" not in out:
        out["kept_idx"] = torch.empty((B, shape.keep), dtype=torch.int32, device=dev)
    if want_scores and "scores" not in out:
        out["scores"] = torch.empty((B, shape.vis_len), dtype=torch.float32, device=dev)
    ho = None
    if not shape.in_place:
        ho = out.get("hidden")
        if ho is None:
            ho = torch.empty((B, So, shape.hidden), dtype=hidden.dtype, device=dev)
    rc = lib().vscan_llm_prune_fused(ctypes.byref(desc), _ptr(hidden), _ptr(w_q), _ptr(w_k_t),
                                     _ptr(out["kept_idx"]), _ptr(ho), _ptr(out.get("scores")),
                                     _ptr(workspace), workspace.numel(), _stream_handle())
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_llm_prune_fused")
    out["hidden"] = hidden[:, :So] if shape.in_place else ho
    out["workspace"] = workspace
    return out


def encoder_fused_workspace_size(desc: EncoderDesc, with_local_triple: bool = False) -> int:
    n = ctypes.c_size_t(0)
    rc = lib().vscan_encoder_fused_workspace_size(ctypes.byref(desc), int(with_local_triple),
                                                  ctypes.byref(n))
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_encoder_fused_workspace_size")
    return int(n.value)


def encoder_reduce_fused(shape, hidden, w_q, w_k_t, x, local=None, want_assign: bool = False,
                         want_scores: bool = False, workspace=None, out=None) -> Dict[str, object]:
    """vscan_encoder_reduce_fused on CUDA bf16 tensors hidden [B,C,S,D] ([CLS] row first), w_q
    [H*dh, D], w_k_t [D, H*dh], x [B,C*N,D]; `local` is an optional (hidden, w_q, w_k_t) triple
    of the shallow layer."""
    import torch
    desc = encoder_desc(shape)
    need = encoder_fused_workspace_size(desc, local is not None)
    dev = hidden.device
    B, T, D = shape.batch, shape.tokens_per_image, shape.feat_dim
    hd = shape.heads * shape.head_dim
    triples = [(hidden, w_q, w_k_t)] + ([tuple(local)] if local is not None else [])
    for h, a, b in triples:
        for t in (h, a, b):
            assert t.is_cuda and t.is_contiguous() and t.dtype == _torch_dtype(shape.dtype)
        assert tuple(h.shape) == (B, shape.n_segments, shape.rows, D)
        assert tuple(a.shape) == (hd, D) and tuple(b.shape) == (D, hd)
    assert x.is_cuda and x.is_contiguous() and tuple(x.shape) == (B, T, D)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    out = dict(out) if out else {}
    if "kept_idx" not in out:
        out["kept_idx"] = torch.empty((B, shape.keep), dtype=torch.int32, device=dev)
    if "merged" not in out:
        out["merged"] = torch.empty((B, shape.keep, D), dtype=x.dtype, device=dev)
    if want_assign and "assign" not in out:
        out["assign"] = torch.empty((B, T), dtype=torch.int32, device=dev)
    if want_scores and "scores" not in out:
        out["scores"] = torch.empty((B, T), dtype=torch.float32, device=dev)
    loc = triples[1] if local is not None else (None, None, None)
    rc = lib().vscan_encoder_reduce_fused(ctypes.byref(desc), _ptr(hidden), _ptr(w_q), _ptr(w_k_t),
                                          _ptr(loc[0]), _ptr(loc[1]), _ptr(loc[2]), _ptr(x),
                                          _ptr(out["kept_idx"]), _ptr(out["merged"]),
                                          _ptr(out.get("assign")), _ptr(out.get("scores")),
                                          _ptr(workspace), workspace.numel(), _stream_handle())
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_encoder_reduce_fused")
    out["workspace"] = workspace
    return out


def llm_prune_fused_ragged(shape, meta, hidden, w_q, w_k_t, want_scores: bool = False) -> Dict[str, object]:
    """vscan_llm_prune_fused_ragged.  `shape` carries the shared fields and the capacities;
    `meta` lists (seq_len, vis_start, vis_len, keep) per sequence.  The out-of-place result is
    shaped like `hidden` (zero-filled here past a sequence's result); `out_len` lists the
    result lengths."""
    import torch
    desc = llm_desc(shape)
    need = llm_fused_workspace_size(desc)
    dev = hidden.device
    B = shape.batch
    assert len(meta) == B
    host = (ctypes.c_int32 * (4 * max(B, 1)))(*[int(x) for m in meta for x in m])
    meta_dev = torch.tensor([list(map(int, m)) for m in meta], dtype=torch.int32,
                            device=dev).reshape(B, 4).contiguous()
    workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    out = {"kept_idx": torch.empty((B, shape.keep), dtype=torch.int32, device=dev)}
    if want_scores:
        out["scores"] = torch.zeros((B, shape.vis_len), dtype=torch.float32, device=dev)
    ho = None if shape.in_place else torch.zeros_like(hidden)
    rc = lib().vscan_llm_prune_fused_ragged(ctypes.byref(desc), ctypes.cast(host, ctypes.c_void_p),
                                            _ptr(meta_dev), _ptr(hidden), _ptr(w_q), _ptr(w_k_t),
                                            _ptr(out["kept_idx"]), _ptr(ho), _ptr(out.get("scores")),
                                            _ptr(workspace), workspace.numel(), _stream_handle())
    if rc != VSCAN_OK:
        raise VscanError(rc, "vscan_llm_prune_fused_ragged")
    out["hidden"] = hidden if shape.in_place else ho
    out["out_len"] = [m[0] - m[2] + m[3] for m in meta]
    out["meta_device"], out["workspace"] = meta_dev, workspace  # alive until the work has run
    return out
