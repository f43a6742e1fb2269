"""Runs inside a child process whose runtime has AddressSanitizer preloaded (started by
tests/test_sanitized_host.py, never collected by pytest).  argv: the sanitized oracle library,
the sanitized CPU build of the host layer.  Exercises the C oracle on small seeded inputs and
every entry point of the host layer, good and bad descriptors alike, with stand-in launchers
that check the scratch regions handed to them.  Prints one line `sanitized-ok ...` at the end."""
import ctypes
import dataclasses
import sys

import numpy as np

oracle_lib, host_lib = sys.argv[1], sys.argv[2]

from oracle import vscan_oracle as vo  # noqa: E402
vo._LIB = oracle_lib          # the oracle's loader takes the library from this path
vo._lib = None
from paper_2505_22654_amd import binding as vb  # noqa: E402
from paper_2505_22654_amd import workloads as wl  # noqa: E402

# ---- oracle: both score modes, windows that do not divide the grid, fused and ragged-tail sizes
enc = wl.EncoderShape(dtype=wl.F32, batch=2, n_segments=2, grid_h=5, grid_w=7, has_cls=1,
                      score_mode=0, heads=3, head_dim=8, feat_dim=24, win_rows=2, win_cols=3,
                      keep_global=3, keep_local=7)
for mode, dom in ((0, 0), (0, 1), (1, 0)):
    s = dataclasses.replace(enc, score_mode=mode, softmax_domain=dom)
    inp = wl.encoder_inputs(s, 11)
    ref = vo.encoder_reduce(s, inp["q"], inp["k"], inp["x"])
    assert ref["kept"].shape == (2, 2 * 10) and np.isfinite(ref["merged"]).all()
llm = wl.LlmShape(dtype=wl.BF16, batch=3, prefix=2, vis_len=37, text=5, n_query=2, q_heads=4,
                  kv_heads=2, head_dim=16, hidden=24, keep=9, in_place=0, softmax_domain=1)
inp = wl.llm_inputs(llm, 12)
ref = vo.llm_prune(llm, inp["q"], inp["k"], inp["v"], inp["hidden"])
assert ref["kept"].shape == (3, 9)
w = wl.llm_weights(llm, 13)
ref = vo.llm_prune_fused(llm, inp["hidden"], w["w_q"], w["w_k"])
assert ref["kept"].shape == (3, 9)
ehid = wl.encoder_hidden_inputs(enc, 14)
ref = vo.encoder_reduce_fused(dataclasses.replace(enc, dtype=wl.BF16), ehid["hidden"], ehid["w_q"],
                              ehid["w_k"], ehid["x"])
assert ref["kept"].shape == (2, 20)

# ---- host layer (argument types as in the binding; the static-scratch entry is GPU code and
# not part of this build)
L = ctypes.CDLL(host_lib)
vp, szp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t)
L.vscan_encoder_workspace_size.argtypes = [ctypes.POINTER(vb.EncoderDesc), ctypes.c_int, szp]
L.vscan_encoder_fused_workspace_size.argtypes = [ctypes.POINTER(vb.EncoderDesc), ctypes.c_int, szp]
L.vscan_llm_workspace_size.argtypes = [ctypes.POINTER(vb.LlmDesc), szp]
L.vscan_llm_fused_workspace_size.argtypes = [ctypes.POINTER(vb.LlmDesc), szp]
L.vscan_encoder_reduce.argtypes = [ctypes.POINTER(vb.EncoderDesc)] + [vp] * 10 + [ctypes.c_size_t, vp]
L.vscan_encoder_reduce_fused.argtypes = ([ctypes.POINTER(vb.EncoderDesc)] + [vp] * 12 +
                                        [ctypes.c_size_t, vp])
L.vscan_llm_prune.argtypes = [ctypes.POINTER(vb.LlmDesc)] + [vp] * 10 + [ctypes.c_size_t, vp]
L.vscan_llm_prune_fused.argtypes = [ctypes.POINTER(vb.LlmDesc)] + [vp] * 7 + [ctypes.c_size_t, vp]
L.vscan_llm_prune_ragged.argtypes = [ctypes.POINTER(vb.LlmDesc)] + [vp] * 12 + [ctypes.c_size_t, vp]
L.vscan_llm_prune_fused_ragged.argtypes = ([ctypes.POINTER(vb.LlmDesc)] + [vp] * 9 +
                                           [ctypes.c_size_t, vp])
L.vscan_test_window.argtypes = [vp, ctypes.c_size_t]
L.vscan_test_report.argtypes = [ctypes.POINTER(ctypes.c_int)] * 3
L.vscan_status_string.restype = ctypes.c_char_p

FAKE = 0x7F0000001000      # user tensors: aligned, outside every window, never dereferenced
WS = 0x500000000000        # workspace base: aligned, never dereferenced


def size(fn, desc, *more):
    n = ctypes.c_size_t(0)
    rc = fn(ctypes.byref(desc), *more, ctypes.byref(n))
    return rc, n.value


ok = bad = 0
for idx in (1, 2, 3, 4, 5, 6):
    cfg = wl.config(idx)
    e, l = cfg.encoder, cfg.llm
    variants = [e, dataclasses.replace(e, batch=0)] if e is not None else []
    if e is not None and e.has_cls:
        variants.append(dataclasses.replace(e, softmax_domain=1))
    for shape in variants:
        d = vb.encoder_desc(shape)
        for with_local in (0, 1):
            rc, n = size(L.vscan_encoder_workspace_size, d, with_local)
            assert rc == 0 and n % 256 == 0, (idx, rc)
            L.vscan_test_window(WS, n)
            loc = FAKE if with_local else None
            rc = L.vscan_encoder_reduce(ctypes.byref(d), FAKE, FAKE, loc, loc, FAKE, FAKE, FAKE, FAKE,
                                        FAKE, WS, n, None)
            assert rc == 0, (idx, vb.status_string(rc) if False else rc)
            ok += 1
            # one byte short, misaligned, missing
            assert L.vscan_encoder_reduce(ctypes.byref(d), FAKE, FAKE, loc, loc, FAKE, FAKE, FAKE, None,
                                          None, WS, n - 1, None) == vb.VSCAN_ERR_WORKSPACE
            assert L.vscan_encoder_reduce(ctypes.byref(d), FAKE, FAKE, loc, loc, FAKE, FAKE, FAKE, None,
                                          None, WS + 8, n + 8, None) == vb.VSCAN_ERR_ALIGN
            bad += 2
        # [CLS] scoring and mean attention from hidden states, both element types
        for with_local in (0, 1):
            rc, n = size(L.vscan_encoder_fused_workspace_size, d, with_local)
            if rc == vb.VSCAN_ERR_UNSUPPORTED:
                continue
            assert rc == 0
            L.vscan_test_window(WS, n)
            loc = FAKE if with_local else None
            rc = L.vscan_encoder_reduce_fused(ctypes.byref(d), FAKE, FAKE, FAKE, loc, loc, loc, FAKE,
                                              FAKE, FAKE, FAKE, FAKE, WS, n, None)
            assert rc == 0, (idx, rc)
            ok += 1
    for shape in ((l, dataclasses.replace(l, in_place=1), dataclasses.replace(l, softmax_domain=1),
                   dataclasses.replace(l, keep=0), dataclasses.replace(l, batch=0)) if l is not None else ()):
        d = vb.llm_desc(shape)
        rc, n = size(L.vscan_llm_workspace_size, d)
        assert rc == 0 and n % 256 == 0
        L.vscan_test_window(WS, n)
        outs = [None] * 3 if shape.in_place else [FAKE] * 3
        rc = L.vscan_llm_prune(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, *outs, FAKE, WS, n, None)
        assert rc == 0, (idx, rc)
        ok += 1
        meta = (ctypes.c_int32 * (4 * max(shape.batch, 1)))()
        for b in range(shape.batch):
            meta[4 * b:4 * b + 4] = [shape.seq_len - b % 2, shape.vis_start, shape.vis_len - b % 2,
                                     max(shape.keep - b % 2, 0)]
        rc = L.vscan_llm_prune_ragged(ctypes.byref(d), ctypes.addressof(meta), FAKE, FAKE, FAKE, FAKE,
                                      FAKE, FAKE, *outs, FAKE, WS, n, None)
        assert rc == 0, (idx, rc)
        ok += 1
        # both element types
        rc, n = size(L.vscan_llm_fused_workspace_size, d)
        if rc == 0:
            L.vscan_test_window(WS, n)
            ho = None if shape.in_place else FAKE
            assert L.vscan_llm_prune_fused(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, ho, FAKE, WS, n,
                                           None) == 0
            assert L.vscan_llm_prune_fused_ragged(ctypes.byref(d), ctypes.addressof(meta), FAKE, FAKE,
                                                  FAKE, FAKE, FAKE, ho, FAKE, WS, n, None) == 0
            ok += 2
        else:
            assert rc == vb.VSCAN_ERR_UNSUPPORTED, rc

# descriptors that must be refused: nothing may reach a launcher
calls0 = ctypes.c_int(0); regions = ctypes.c_int(0); viol = ctypes.c_int(0)
L.vscan_test_report(ctypes.byref(calls0), ctypes.byref(regions), ctypes.byref(viol))
e1 = wl.config(1).encoder
for change in (dict(batch=-1), dict(grid_h=0), dict(head_dim=60), dict(feat_dim=1001), dict(win_rows=25),
               dict(keep_global=-1), dict(keep_local=10 ** 6), dict(grid_h=2 ** 15, grid_w=2 ** 15),
               dict(batch=2 ** 30, n_segments=2 ** 30), dict(heads=2 ** 30)):
    d = vb.encoder_desc(dataclasses.replace(e1, **change))
    rc, _ = size(L.vscan_encoder_workspace_size, d, 0)
    assert rc < 0, change
    assert L.vscan_encoder_reduce(ctypes.byref(d), FAKE, FAKE, None, None, FAKE, FAKE, FAKE, None, None,
                                  WS, 1 << 40, None) < 0
    bad += 1
l1 = wl.config(1).llm
for change in (dict(batch=-1), dict(vis_len=0), dict(keep=10 ** 6), dict(head_dim=12), dict(q_heads=5),
               dict(prefix=2 ** 30, vis_len=2 ** 30, text=2 ** 30), dict(batch=2 ** 30, kv_heads=2 ** 30,
                                                                         q_heads=2 ** 30)):
    try:
        d = vb.llm_desc(dataclasses.replace(l1, **change))
    except (OverflowError, TypeError):
        continue
    rc, _ = size(L.vscan_llm_workspace_size, d)
    assert rc < 0, change
    assert L.vscan_llm_prune(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, WS,
                             1 << 40, None) < 0
    bad += 1
calls = ctypes.c_int(0)
L.vscan_test_report(ctypes.byref(calls), ctypes.byref(regions), ctypes.byref(viol))
assert calls.value == calls0.value, "a refused descriptor reached a launcher"
assert viol.value == 0, f"{viol.value} scratch regions outside the workspace, unaligned or overlapping"
assert calls.value > 100 and regions.value > 300
print(f"sanitized-ok entry-point calls {ok}, refused {bad}, launcher calls {calls.value}, "
      f"regions checked {regions.value}")
