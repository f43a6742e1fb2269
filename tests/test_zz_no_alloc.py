"""vscan_llm_prune_static (the entry point that allocates nothing: its scratch is a fixed array
inside the library) against vscan_llm_prune on the same inputs, through the C ABI."""
import ctypes
import dataclasses

import numpy as np
import pytest

from paper_2505_22654_amd import binding as vb
from paper_2505_22654_amd import workloads as wl
from tests import parity_utils as pu

FAKE = 0x7F0000001000  # aligned, never dereferenced


def _shape(**kw):
    base = dict(dtype=wl.BF16, batch=3, prefix=7, vis_len=700, text=33, n_query=2, q_heads=8,
                kv_heads=4, head_dim=64, hidden=256, keep=200)
    base.update(kw)
    return wl.LlmShape(**base)


def test_static_scratch_limit_is_enforced_on_the_host():
    """A request beyond the fixed scratch is refused before anything touches the GPU."""
    big = _shape(batch=64, vis_len=20000, kv_heads=4, q_heads=4, keep=10)
    desc = vb.llm_desc(big)
    assert vb.llm_workspace_size(desc) > vb.STATIC_SCRATCH_BYTES
    rc = vb.lib().vscan_llm_prune_static(ctypes.byref(desc), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                         FAKE, FAKE, None, None)
    assert rc == vb.VSCAN_ERR_WORKSPACE
    # descriptor and pointer errors come out as for vscan_llm_prune
    bad = vb.llm_desc(_shape(keep=701))
    rc = vb.lib().vscan_llm_prune_static(ctypes.byref(bad), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                         FAKE, FAKE, None, None)
    assert rc == vb.VSCAN_ERR_BUDGET
    ok = vb.llm_desc(_shape())
    rc = vb.lib().vscan_llm_prune_static(ctypes.byref(ok), None, FAKE, FAKE, FAKE, FAKE, FAKE,
                                         FAKE, FAKE, None, None)
    assert rc == vb.VSCAN_ERR_NULL


@pytest.mark.gpu
def test_static_scratch_matches_workspace_entry_point():
    """Two calls in a row, the second on a smaller input (the scratch still holds the first
    call's partial scores), each compared with vscan_llm_prune and with the oracle."""
    import torch
    for shape, seed in ((_shape(), 6100), (_shape(batch=2, vis_len=150, text=9, keep=40), 6200),
                        (_shape(in_place=1, batch=2, vis_len=1300, keep=17), 6300)):
        inp, ref, info = pu.screened_llm_case(shape, seed=seed)
        dev = [pu.to_device(inp[n], shape.dtype) for n in ("q", "k", "v", "hidden")]
        dev2 = [t.clone() for t in dev]
        got = vb.llm_prune(shape, *dev, want_scores=True, static_scratch=True)
        want = vb.llm_prune(shape, *dev2, want_scores=True)
        torch.cuda.synchronize()
        for name in ("kept_idx", "scores", "k", "v", "hidden"):
            assert torch.equal(got[name], want[name]), (shape, name)
        print("static", info, pu.check_llm(shape, inp, ref, got, "static"))
