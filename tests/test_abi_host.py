"""Host-only checks of the C ABI: the library loads, exports what include/vscan.h
declares, sizes workspaces and rejects bad descriptors before touching the GPU.

Every negative call here fails validation, so no kernel is ever launched and the
fake pointer values are never dereferenced.
"""
import ctypes
import dataclasses
import os
import re

import pytest

from paper_2505_22654_amd import binding as vb
from paper_2505_22654_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000  # aligned, never dereferenced


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "vscan.h")).read()
    declared = set(re.findall(r"\b(vscan_[a-z0-9_]+)\s*\(", header))
    assert declared == set(vb.EXPORTS)
    L = vb.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_version_and_status_strings():
    assert vb.version() == 0x00010000
    seen = set()
    for code in range(0, -10, -1):
        s = vb.status_string(code)
        assert s and s != "unknown status" and s not in seen
        seen.add(s)
    assert vb.status_string(-99) == "unknown status"


def test_descriptor_layout_matches_header():
    # 17 four-byte fields / 15 four-byte fields, no padding
    assert ctypes.sizeof(vb.EncoderDesc) == 17 * 4
    assert ctypes.sizeof(vb.LlmDesc) == 15 * 4


def test_workspace_sizes_for_the_benchmark_configs():
    sizes = {}
    for i in (1, 2, 3, 4):
        w = wl.config(i)
        n = vb.encoder_workspace_size(vb.encoder_desc(w.encoder))
        n_local = vb.encoder_workspace_size(vb.encoder_desc(w.encoder), True)
        assert 0 < n < n_local and n % 256 == 0
        sizes[i] = n
    assert sizes[1] < sizes[2] < sizes[3]
    for i in (1, 2, 3, 4, 5):
        w = wl.config(i)
        n = vb.llm_workspace_size(vb.llm_desc(w.llm))
        s = w.llm
        assert n >= s.batch * s.kv_heads * s.vis_len * 4 and n % 256 == 0


def _enc_call(desc, q=FAKE, k=FAKE, ql=None, kl=None, x=FAKE, kept=FAKE, merged=FAKE,
              ws=FAKE, ws_bytes=1 << 40):
    return vb.lib().vscan_encoder_reduce(ctypes.byref(desc) if desc is not None else None, q, k,
                                         ql, kl, x, kept, merged, None, None, ws, ws_bytes, None)


def _enc_shape(**kw):
    return dataclasses.replace(wl.config(1).encoder, **kw)


@pytest.mark.parametrize("change,status", [
    (dict(dtype="f32", batch=-1), vb.VSCAN_ERR_SHAPE),
    (dict(grid_h=0), vb.VSCAN_ERR_SHAPE),
    (dict(heads=0), vb.VSCAN_ERR_SHAPE),
    (dict(head_dim=60), vb.VSCAN_ERR_SHAPE),
    (dict(head_dim=264), vb.VSCAN_ERR_SHAPE),
    (dict(feat_dim=1001), vb.VSCAN_ERR_SHAPE),
    (dict(win_rows=25), vb.VSCAN_ERR_SHAPE),
    (dict(has_cls=0), vb.VSCAN_ERR_SHAPE),            # [CLS] scoring without a [CLS] row
    (dict(has_cls=2), vb.VSCAN_ERR_SHAPE),
    (dict(score_mode=7), vb.VSCAN_ERR_DTYPE),
    (dict(softmax_domain=-1), vb.VSCAN_ERR_DTYPE),
    (dict(keep_global=-1), vb.VSCAN_ERR_BUDGET),
    (dict(keep_global=0, keep_local=0), vb.VSCAN_ERR_BUDGET),
    (dict(keep_global=570, keep_local=8), vb.VSCAN_ERR_BUDGET),      # more than N
    (dict(keep_local=4 * 145), vb.VSCAN_ERR_BUDGET),                  # 145 per 144-token window
    (dict(feat_dim=16384), vb.VSCAN_ERR_UNSUPPORTED),
    (dict(grid_h=256, grid_w=256, win_rows=1, win_cols=1), vb.VSCAN_ERR_UNSUPPORTED),
])
def test_encoder_rejects_bad_descriptors(change, status):
    desc = vb.encoder_desc(_enc_shape(**change))
    assert _enc_call(desc) == status
    n = ctypes.c_size_t(0)
    assert vb.lib().vscan_encoder_workspace_size(ctypes.byref(desc), 0, ctypes.byref(n)) == status


def test_encoder_rejects_bad_pointers_and_workspace():
    desc = vb.encoder_desc(_enc_shape())
    need = vb.encoder_workspace_size(desc)
    assert _enc_call(None) == vb.VSCAN_ERR_NULL
    bad = vb.encoder_desc(_enc_shape())
    bad.struct_size = 12
    assert _enc_call(bad) == vb.VSCAN_ERR_VERSION
    bad = vb.encoder_desc(_enc_shape())
    bad.dtype = 5
    assert _enc_call(bad) == vb.VSCAN_ERR_DTYPE
    assert _enc_call(desc, q=None) == vb.VSCAN_ERR_NULL
    assert _enc_call(desc, merged=None) == vb.VSCAN_ERR_NULL
    assert _enc_call(desc, ql=FAKE, kl=None) == vb.VSCAN_ERR_NULL    # half of the local pair
    assert _enc_call(desc, x=FAKE + 8) == vb.VSCAN_ERR_ALIGN
    assert _enc_call(desc, kept=FAKE + 2) == vb.VSCAN_ERR_ALIGN
    assert _enc_call(desc, ws=None) == vb.VSCAN_ERR_WORKSPACE
    assert _enc_call(desc, ws_bytes=need - 1) == vb.VSCAN_ERR_WORKSPACE
    assert _enc_call(desc, ws=FAKE + 4) == vb.VSCAN_ERR_ALIGN
    # the local pair needs a larger workspace than the plain call
    assert _enc_call(desc, ql=FAKE, kl=FAKE, ws_bytes=need) == vb.VSCAN_ERR_WORKSPACE
    assert vb.lib().vscan_encoder_workspace_size(ctypes.byref(desc), 0, None) == vb.VSCAN_ERR_NULL


def test_empty_batch_is_a_no_op():
    desc = vb.encoder_desc(_enc_shape(batch=0))
    assert _enc_call(desc) == vb.VSCAN_OK
    ldesc = vb.llm_desc(dataclasses.replace(wl.config(1).llm, batch=0))
    assert _llm_call(ldesc) == vb.VSCAN_OK


def _llm_call(desc, q=FAKE, k=FAKE, v=FAKE, hidden=FAKE, kept=FAKE, ko=FAKE, vo=FAKE, ho=FAKE,
              ws=FAKE, ws_bytes=1 << 40):
    return vb.lib().vscan_llm_prune(ctypes.byref(desc) if desc is not None else None, q, k, v,
                                    hidden, kept, ko, vo, ho, None, ws, ws_bytes, None)


def _llm_shape(**kw):
    return dataclasses.replace(wl.config(1).llm, **kw)


@pytest.mark.parametrize("change,status", [
    (dict(vis_len=0), vb.VSCAN_ERR_SHAPE),
    (dict(n_query=0), vb.VSCAN_ERR_SHAPE),
    (dict(n_query=41), vb.VSCAN_ERR_SHAPE),            # queries would overlap the visual span
    (dict(q_heads=30), vb.VSCAN_ERR_SHAPE),            # not a multiple of kv_heads
    (dict(head_dim=100), vb.VSCAN_ERR_SHAPE),
    (dict(hidden=4100), vb.VSCAN_ERR_SHAPE),
    (dict(in_place=3), vb.VSCAN_ERR_SHAPE),
    (dict(softmax_domain=2), vb.VSCAN_ERR_DTYPE),
    (dict(keep=65), vb.VSCAN_ERR_BUDGET),
    (dict(keep=-1), vb.VSCAN_ERR_BUDGET),
    (dict(kv_heads=1, n_query=3), vb.VSCAN_ERR_UNSUPPORTED),   # 96 query rows per kv head
    (dict(prefix=0, vis_len=60000, text=8, keep=10), vb.VSCAN_ERR_UNSUPPORTED),
])
def test_llm_rejects_bad_descriptors(change, status):
    desc = vb.llm_desc(_llm_shape(**change))
    assert _llm_call(desc) == status
    n = ctypes.c_size_t(0)
    assert vb.lib().vscan_llm_workspace_size(ctypes.byref(desc), ctypes.byref(n)) == status


def test_llm_rejects_bad_pointers_and_workspace():
    desc = vb.llm_desc(_llm_shape())
    need = vb.llm_workspace_size(desc)
    assert _llm_call(None) == vb.VSCAN_ERR_NULL
    assert _llm_call(desc, hidden=None) == vb.VSCAN_ERR_NULL
    assert _llm_call(desc, ko=None) == vb.VSCAN_ERR_NULL             # out of place needs outputs
    assert _llm_call(desc, v=FAKE + 4) == vb.VSCAN_ERR_ALIGN
    assert _llm_call(desc, ws_bytes=need - 1) == vb.VSCAN_ERR_WORKSPACE
    inplace = vb.llm_desc(_llm_shape(in_place=1))
    assert _llm_call(inplace) == vb.VSCAN_ERR_NULL                   # in place forbids outputs
    assert _llm_call(inplace, ko=None, vo=None, ho=None, ws=None) == vb.VSCAN_ERR_WORKSPACE


def _ragged_call(desc, rows, meta_dev=FAKE, **kw):
    host = (ctypes.c_int32 * (4 * max(len(rows), 1)))(*[x for r in rows for x in r])
    a = dict(q=FAKE, k=FAKE, v=FAKE, hidden=FAKE, kept=FAKE, ko=FAKE, vo=FAKE, ho=FAKE, ws=FAKE)
    a.update(kw)
    return vb.lib().vscan_llm_prune_ragged(
        ctypes.byref(desc), ctypes.cast(host, ctypes.c_void_p) if rows is not None else None,
        meta_dev, a["q"], a["k"], a["v"], a["hidden"], a["kept"], a["ko"], a["vo"], a["ho"], None,
        a["ws"], 1 << 40, None)


@pytest.mark.parametrize("row,status", [
    ((140, 35, 64, 32), vb.VSCAN_ERR_SHAPE),    # longer than the capacity (139 rows)
    ((0, 0, 1, 0), vb.VSCAN_ERR_SHAPE),
    ((139, -1, 64, 32), vb.VSCAN_ERR_SHAPE),
    ((139, 35, 0, 0), vb.VSCAN_ERR_SHAPE),      # no visual token
    ((139, 35, 65, 32), vb.VSCAN_ERR_SHAPE),    # span longer than the capacity (64)
    ((100, 40, 60, 10), vb.VSCAN_ERR_SHAPE),    # no room for the query position after the span
    ((139, 35, 64, 33), vb.VSCAN_ERR_BUDGET),   # above the index capacity (32)
    ((139, 35, 20, 21), vb.VSCAN_ERR_BUDGET),   # more than the sequence has
    ((139, 35, 64, -1), vb.VSCAN_ERR_BUDGET),
])
def test_ragged_rejects_bad_sequences(row, status):
    desc = vb.llm_desc(_llm_shape(batch=2))
    good = (139, 35, 64, 32)
    assert _ragged_call(desc, [good, row]) == status


def test_ragged_pointer_checks_and_empty_batch():
    desc = vb.llm_desc(_llm_shape(batch=1))
    good = [(139, 35, 64, 32)]
    assert _ragged_call(desc, good, meta_dev=None) == vb.VSCAN_ERR_NULL
    assert _ragged_call(desc, good, meta_dev=FAKE + 2) == vb.VSCAN_ERR_ALIGN
    assert _ragged_call(desc, good, hidden=None) == vb.VSCAN_ERR_NULL
    assert _ragged_call(desc, good, ko=None) == vb.VSCAN_ERR_NULL
    assert _ragged_call(desc, good, ws=None) == vb.VSCAN_ERR_WORKSPACE
    empty = vb.llm_desc(_llm_shape(batch=0))
    assert _ragged_call(empty, [], meta_dev=None) == vb.VSCAN_OK      # nothing to enqueue
    # the capacities themselves go through the same checks as a uniform descriptor
    assert _ragged_call(vb.llm_desc(_llm_shape(head_dim=100)), good) == vb.VSCAN_ERR_SHAPE


def _fused_llm_call(desc, hidden=FAKE, wq=FAKE, wkt=FAKE, kept=FAKE, ho=FAKE, ws=FAKE,
                    ws_bytes=1 << 40):
    return vb.lib().vscan_llm_prune_fused(ctypes.byref(desc) if desc is not None else None, hidden,
                                          wq, wkt, kept, ho, None, ws, ws_bytes, None)


def _fused_enc_call(desc, hidden=FAKE, wq=FAKE, wkt=FAKE, local=(None, None, None), x=FAKE,
                    kept=FAKE, merged=FAKE, ws=FAKE, ws_bytes=1 << 40):
    return vb.lib().vscan_encoder_reduce_fused(ctypes.byref(desc) if desc is not None else None,
                                               hidden, wq, wkt, local[0], local[1], local[2], x,
                                               kept, merged, None, None, ws, ws_bytes, None)


def test_fused_entry_points_validate_on_the_host():
    """Scoring from hidden states: the usual pointer, alignment and workspace checks; every
    call here fails one of them (or has an empty batch), so nothing is launched."""
    bf = lambda sh: dataclasses.replace(sh, dtype=wl.BF16)
    ldesc = vb.llm_desc(bf(_llm_shape()))
    need = vb.llm_fused_workspace_size(ldesc)
    assert need > vb.llm_workspace_size(ldesc)
    assert _fused_llm_call(None) == vb.VSCAN_ERR_NULL
    assert vb.llm_fused_workspace_size(vb.llm_desc(_llm_shape())) > 0                  # fp32 is served
    assert _fused_llm_call(vb.llm_desc(_llm_shape()), ws_bytes=16) == vb.VSCAN_ERR_WORKSPACE
    assert _fused_llm_call(vb.llm_desc(bf(_llm_shape(head_dim=100)))) == vb.VSCAN_ERR_SHAPE
    assert _fused_llm_call(vb.llm_desc(bf(_llm_shape(keep=65)))) == vb.VSCAN_ERR_BUDGET
    assert _fused_llm_call(ldesc, wq=None) == vb.VSCAN_ERR_NULL
    assert _fused_llm_call(ldesc, ho=None) == vb.VSCAN_ERR_NULL                        # out of place
    assert _fused_llm_call(vb.llm_desc(bf(_llm_shape(in_place=1)))) == vb.VSCAN_ERR_NULL   # ho given
    assert _fused_llm_call(ldesc, wkt=FAKE + 8) == vb.VSCAN_ERR_ALIGN
    assert _fused_llm_call(ldesc, ws_bytes=need - 1) == vb.VSCAN_ERR_WORKSPACE
    assert _fused_llm_call(vb.llm_desc(bf(_llm_shape(batch=0)))) == vb.VSCAN_OK
    # 4 GiB of hidden states and more: byte offsets no longer fit the kernels' 32-bit row offsets
    big = bf(_llm_shape(batch=64, prefix=0, vis_len=8192, text=8, keep=10))
    assert _fused_llm_call(vb.llm_desc(big)) == vb.VSCAN_ERR_UNSUPPORTED

    edesc = vb.encoder_desc(bf(_enc_shape()))
    eneed = vb.encoder_fused_workspace_size(edesc)
    assert eneed > vb.encoder_workspace_size(edesc)
    assert vb.encoder_fused_workspace_size(edesc, True) > eneed
    assert vb.encoder_fused_workspace_size(vb.encoder_desc(_enc_shape())) > 0            # fp32 is served
    assert _fused_enc_call(vb.encoder_desc(_enc_shape()), ws_bytes=16) == vb.VSCAN_ERR_WORKSPACE
    # mean-attention scoring is served (Q and K projected in fp32): larger scratch, and heads
    # wider than 512 bytes in fp32 are refused
    mean = bf(_enc_shape(has_cls=0, score_mode=1))
    assert vb.encoder_fused_workspace_size(vb.encoder_desc(mean)) > vb.encoder_workspace_size(vb.encoder_desc(mean))
    wide = bf(_enc_shape(has_cls=0, score_mode=1, head_dim=136))
    assert _fused_enc_call(vb.encoder_desc(wide)) == vb.VSCAN_ERR_UNSUPPORTED
    assert _fused_enc_call(edesc, local=(FAKE, FAKE, None)) == vb.VSCAN_ERR_NULL       # partial triple
    assert _fused_enc_call(edesc, x=None) == vb.VSCAN_ERR_NULL
    assert _fused_enc_call(edesc, hidden=FAKE + 4) == vb.VSCAN_ERR_ALIGN
    assert _fused_enc_call(edesc, ws_bytes=eneed - 1) == vb.VSCAN_ERR_WORKSPACE
    assert _fused_enc_call(edesc, local=(FAKE, FAKE, FAKE), ws_bytes=eneed) == vb.VSCAN_ERR_WORKSPACE
    assert _fused_enc_call(vb.encoder_desc(bf(_enc_shape(batch=0)))) == vb.VSCAN_OK


def test_fused_ragged_validates_the_table_on_the_host():
    desc = vb.llm_desc(dataclasses.replace(_llm_shape(batch=2), dtype=wl.BF16))

    def call(rows, meta_dev=FAKE, hidden=FAKE, ho=FAKE, ws=FAKE):
        host = (ctypes.c_int32 * (4 * max(len(rows), 1)))(*[x for r in rows for x in r])
        return vb.lib().vscan_llm_prune_fused_ragged(ctypes.byref(desc), host, meta_dev, hidden, FAKE,
                                                     FAKE, FAKE, ho, None, ws, 1 << 40, None)
    good = (139, 35, 64, 32)
    assert call([good, (140, 35, 64, 32)]) == vb.VSCAN_ERR_SHAPE     # longer than the capacity
    assert call([good, (139, 35, 65, 32)]) == vb.VSCAN_ERR_SHAPE     # span beyond the capacity
    assert call([good, (99, 35, 64, 32)]) == vb.VSCAN_ERR_SHAPE      # span and query overlap
    assert call([good, (139, 35, 64, 33)]) == vb.VSCAN_ERR_BUDGET    # budget beyond the capacity
    assert call([good, good], meta_dev=None) == vb.VSCAN_ERR_NULL
    assert call([good, good], meta_dev=FAKE + 2) == vb.VSCAN_ERR_ALIGN
    assert call([good, good], hidden=None) == vb.VSCAN_ERR_NULL
    assert call([good, good], ho=None) == vb.VSCAN_ERR_NULL
    assert call([good, good], ws=None) == vb.VSCAN_ERR_WORKSPACE


def test_binding_fails_loudly_without_the_library(monkeypatch):
    monkeypatch.setattr(vb, "_lib", None)
    monkeypatch.setattr(vb, "LIB_PATH", "/nonexistent/libvscan.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        vb.lib()
