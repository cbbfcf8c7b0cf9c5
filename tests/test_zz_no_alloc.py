"""The entry point that allocates nothing: sp_pool_select_static (scratch space inside the
library's device image) against sp_pool_select (caller's workspace) and the oracle, on two calls in
a row, the second with a smaller input -- the shared scratch then still holds the first call's data."""
import ctypes as C

import numpy as np
import pytest

from oracle import specprefill_oracle as orc
from paper_2502_02789_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _both(scores, cu, chunk, window, rate):
    """-> (kept, cu_keep, chunk scores) of the workspace entry point and of the static one"""
    import torch
    from paper_2502_02789_amd import binding as sp, device as dev
    sc = torch.from_numpy(scores).cuda()
    cu_d = torch.from_numpy(cu).cuda()
    out = []
    for static in (False, True):
        sel = dev.Selector(sc, cu_d, chunk=chunk, pool_window=window, keep_rate=rate, want_chunk_scores=True)
        if static:
            sel.args.d_workspace = None       # the static variant must not need (or touch) a workspace
            sel.args.workspace_bytes = 0
            sp.sp_pool_select_static(sel.args)
        else:
            sel.run()
        torch.cuda.synchronize()
        n = int(sel.cu_keep[-1])
        out.append((sel.kept_idx.cpu().numpy(), sel.cu_keep.cpu().numpy(), sel.chunk_scores.cpu().numpy(), n))
    return out


@pytest.mark.parametrize("lens_pair", [((32768,), (5003,)), ((300, 0, 1, 65, 64, 129, 4000), (700, 33))])
def test_static_scratch_entry_point_equals_the_workspace_one(lens_pair):
    for call, lens in enumerate(lens_pair):        # the second call is the smaller one
        cu = np.zeros(len(lens) + 1, dtype=np.int32)
        cu[1:] = np.cumsum(lens)
        scores = synth.random_scores(100 + call, int(cu[-1]), ties=(call == 1))
        (kept_w, cuk_w, cs_w, n_w), (kept_s, cuk_s, cs_s, n_s) = _both(scores, cu, 32, 13, 0.3)
        assert n_w == n_s and cuk_w.tolist() == cuk_s.tolist()
        assert (kept_w == kept_s).all()                                    # including the untouched tail (-1)
        assert (cs_w.view(np.uint32) == cs_s.view(np.uint32)).all()
        kept_o, cuk_o, _, _ = orc.pool_select(scores, cu, 32, 13, 0.3)
        assert cuk_s.tolist() == cuk_o.tolist() and (kept_s[:n_s] == kept_o).all()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch
    from paper_2502_02789_amd import binding as sp, device as dev
    T = (sp.SP_STATIC_MAX_CHUNKS + 5) * 1              # chunk = 1: more chunks than the scratch holds
    sc = torch.zeros(T, dtype=torch.float32, device="cuda")
    cu_d = torch.tensor([0, T], dtype=torch.int32, device="cuda")
    sel = dev.Selector(sc, cu_d, chunk=1, pool_window=1, keep_rate=0.5)
    sel.kept_idx.fill_(-9)
    lib = sp.load_library()
    assert lib.sp_pool_select_static(C.byref(sel.args), None) == sp.SP_EUNSUPPORTED
    torch.cuda.synchronize()
    assert (sel.kept_idx == -9).all()
    sel.run()                                           # the workspace entry point takes it
    torch.cuda.synchronize()
    assert int(sel.cu_keep[1]) == T // 2 + (T % 2)
