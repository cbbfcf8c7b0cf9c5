"""GPU parity of sp_score_pool_select (one short prompt scored and selected in a single launch)
against the oracle, and against the separate calls."""
import ctypes as C
import math

import numpy as np
import pytest

from oracle import specprefill_oracle as orc
from paper_2502_02789_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _run_fused(w, inp, mode, chunk, window, rate, n_valid=None, head_major=False):
    import torch
    from paper_2502_02789_amd import device as dev
    q = dev.bf16_from_bits(inp["q"])
    if head_major:
        ks = [dev.bf16_from_bits(np.ascontiguousarray(k.transpose(1, 0, 2))).permute(1, 0, 2) for k in inp["k"]]
    else:
        ks = [dev.bf16_from_bits(k) for k in inp["k"]]
    cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
    nv = None if n_valid is None else torch.tensor([n_valid], dtype=torch.int32, device="cuda")
    s = dev.Scorer(q, ks, cu, H_kv=w.H_kv, scale=1.0 / math.sqrt(w.d), layer_reduce=mode, n_valid=nv, want_lse=True)
    sel = dev.Selector(s.scores, cu, chunk=chunk, pool_window=window, keep_rate=rate, want_chunk_scores=True)
    s.scores.fill_(float("nan"))
    dev.score_pool_select(s, sel)
    torch.cuda.synchronize()
    return s, sel


@pytest.mark.parametrize("mode", [orc.LAYER_MAX, orc.LAYER_MEAN])
@pytest.mark.parametrize("case", [
    dict(number=1),                                                    # the tiny workload as it is
    dict(number=1, seqlens=(2048,), L=3),                              # as many keys as one workgroup takes
    dict(number=1, seqlens=(1,)),                                      # a single key
    dict(number=1, seqlens=(1333,), H=8, H_kv=2, N=2, n_valid=1),      # eight rows per KV head, one valid query
    dict(number=3, seqlens=(777,), L=2, H=8, H_kv=8, N=8, n_valid=5),  # head dim 128, one head per KV head
    dict(number=1, seqlens=(1100,), H=8, H_kv=1, N=2, n_valid=2),      # sixteen rows: every column of the operand
    dict(number=3, seqlens=(2000,), L=2, H=4, H_kv=2, N=3, n_valid=2), # head dim 128, six rows
    dict(number=1, seqlens=(333,), L=5, H=6, H_kv=2, N=4, n_valid=3),  # three heads per KV head, more pairs than waves take at once
    dict(number=1, seqlens=(600,), H=4, H_kv=1, N=1, chunk=1, window=1, rate=0.1),   # the raw variant
    dict(number=1, seqlens=(1500,), chunk=48, window=7, rate=0.33, head_major=True),
])
def test_fused_short_prompt_against_oracle(case, mode):
    case = dict(case)
    number = case.pop("number")
    n_valid = case.pop("n_valid", None)
    head_major = case.pop("head_major", False)
    base = synth.workload(number)
    chunk, window, rate = case.pop("chunk", base.chunk), case.pop("window", base.pool_window), case.pop("rate", base.keep_rate)
    w = synth.scaled(base, salient_frac=0.02, salient_run=1, **case) if case else base
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    nv = None if n_valid is None else np.array([n_valid], dtype=np.int32)
    want, want_lse = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, mode, nv)
    s, sel = _run_fused(w, inp, mode, chunk, window, rate, n_valid, head_major)
    got = s.scores.cpu().numpy()
    hp.assert_scores_close(got, want, f"fused {w.name} {case} mode={mode}")
    np.testing.assert_allclose(s.lse.cpu().numpy(), want_lse, rtol=0, atol=2e-4)
    # stage-isolated: the oracle's selection on these very scores must be identical
    kept_o, cu_keep_o, cs_o, _ = orc.pool_select(got, inp["cu_seqlens"], chunk, window, rate)
    n = int(sel.cu_keep[1])
    assert sel.cu_keep.cpu().tolist() == cu_keep_o.tolist()
    assert (sel.kept_idx[:n].cpu().numpy() == kept_o).all() and (sel.kept_idx[n:] == -1).all()
    np.testing.assert_array_equal(sel.chunk_scores.cpu().numpy()[:len(cs_o)], cs_o.astype(np.float32))
    # end to end against the oracle's own scores: differences only inside the tolerance window
    hp.selection_matches(sel.kept_idx[:n].cpu().numpy(), sel.cu_keep.cpu().numpy(), want, inp["cu_seqlens"], chunk,
                         window, rate, hp.SCORE_RTOL)


def test_fused_equals_the_separate_calls():
    import torch
    from paper_2502_02789_amd import device as dev
    w = synth.workload(1)
    inp = synth.make_qk(w)
    s, sel = _run_fused(w, inp, orc.LAYER_MAX, w.chunk, w.pool_window, w.keep_rate)
    fused_scores = s.scores.clone()
    fused_kept = sel.kept_idx.clone()
    s.run()
    sel.run()
    torch.cuda.synchronize()
    np.testing.assert_allclose(fused_scores.cpu().numpy(), s.scores.cpu().numpy(), rtol=1e-4, atol=1e-12)
    assert (fused_kept == sel.kept_idx).all()


def test_fused_refuses_what_one_workgroup_cannot_hold():
    import torch
    from paper_2502_02789_amd import binding as sp, device as dev
    lib = sp.load_library()
    for changes in (dict(seqlens=(2049,)), dict(seqlens=(300, 200)), dict(seqlens=(500,), H=8, H_kv=1, N=3),
                    dict(seqlens=(500,), N=9)):
        w = synth.scaled(synth.workload(1), **changes)
        inp = synth.make_qk(w)
        q = dev.bf16_from_bits(inp["q"])
        ks = [dev.bf16_from_bits(k) for k in inp["k"]]
        cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
        s = dev.Scorer(q, ks, cu, H_kv=w.H_kv, scale=0.125)
        sel = dev.Selector(s.scores, cu, chunk=32, pool_window=13, keep_rate=0.25)
        s.scores.fill_(-3.0)
        assert lib.sp_score_pool_select(C.byref(s.args), C.byref(sel.args), None) == sp.SP_EUNSUPPORTED, changes
        torch.cuda.synchronize()
        assert (s.scores == -3.0).all() and (sel.kept_idx == -1).all()
    # mismatched halves are an argument error
    w = synth.workload(1)
    inp = synth.make_qk(w)
    cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
    s = dev.Scorer(dev.bf16_from_bits(inp["q"]), [dev.bf16_from_bits(k) for k in inp["k"]], cu, H_kv=w.H_kv, scale=0.125)
    other = torch.zeros(w.T, dtype=torch.float32, device="cuda")
    sel = dev.Selector(other, cu, chunk=32, pool_window=13, keep_rate=0.25)
    assert lib.sp_score_pool_select(C.byref(s.args), C.byref(sel.args), None) == sp.SP_EINVAL
