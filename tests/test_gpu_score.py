"""GPU parity: sp_score (through the C ABI) against the fp64 oracle, element by element."""
import math

import numpy as np
import pytest

from oracle import specprefill_oracle as orc
from paper_2502_02789_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu

MODES = [orc.LAYER_MAX, orc.LAYER_MEAN]


def _check(w, inp, mode, general, n_valid=None, head_major=False):
    scale = 1.0 / math.sqrt(w.d)
    want, want_lse = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, mode, n_valid)
    got, lse = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, scale, mode, n_valid=n_valid,
                            general=general, head_major=head_major)
    err = hp.assert_scores_close(got, want, f"{w.name} mode={mode} general={general}")
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-4)
    return err


@pytest.mark.parametrize("general", [False, True])
@pytest.mark.parametrize("mode", MODES)
def test_tiny_workload(mode, general):
    w = synth.workload(1)
    _check(w, synth.make_qk(w), mode, general)


@pytest.mark.parametrize("general", [False, True])
@pytest.mark.parametrize("mode", MODES)
def test_1b_shape_several_tiles_and_ragged_tail(mode, general):
    w = synth.scaled(synth.workload(2), seqlens=(2999,), L=3)
    _check(w, synth.make_qk(w), mode, general)


@pytest.mark.parametrize("general", [False, True])
@pytest.mark.parametrize("mode", MODES)
def test_8b_shape_several_tiles_and_ragged_tail(mode, general):
    w = synth.scaled(synth.workload(3), seqlens=(5003,), L=2)
    _check(w, synth.make_qk(w), mode, general)


@pytest.mark.parametrize("general", [False, True])
def test_ragged_batch_with_empty_and_one_token_sequences(general):
    w = synth.scaled(synth.workload(4), seqlens=(300, 0, 1, 65, 64, 129), L=2, salient_frac=0.02, salient_run=1)
    inp = synth.make_qk(w)
    for mode in MODES:
        _check(w, inp, mode, general)


@pytest.mark.parametrize("general", [False, True])
def test_valid_query_counts(general):
    w = synth.scaled(synth.workload(2), seqlens=(200, 333), L=2, N=4)
    inp = synth.make_qk(w)
    for mode in MODES:
        _check(w, inp, mode, general, n_valid=np.array([3, 1], dtype=np.int32))


@pytest.mark.parametrize("shape", [dict(H=8, H_kv=8), dict(H=16, H_kv=2), dict(H=6, H_kv=3, N=16), dict(H=4, H_kv=1, N=3)])
def test_other_head_groupings(shape):
    w = synth.scaled(synth.workload(2), seqlens=(517,), L=2, **shape)
    inp = synth.make_qk(w)
    for general in (False, True):
        _check(w, inp, orc.LAYER_MAX, general)


@pytest.mark.parametrize("general", [False, True])
def test_head_major_k_layout(general):
    w = synth.scaled(synth.workload(3), seqlens=(1000,), L=2)
    _check(w, synth.make_qk(w), orc.LAYER_MAX, general, head_major=True)


def test_identical_keys_give_uniform_scores_on_gpu():
    w = synth.scaled(synth.workload(3), seqlens=(777,), L=2)
    inp = synth.make_qk(w)
    inp["k"] = [np.repeat(k[:1], 777, axis=0) for k in inp["k"]]
    for mode in MODES:
        for general in (False, True):
            got, _ = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, 1.0 / math.sqrt(w.d), mode,
                                  general=general)
            np.testing.assert_allclose(got, 1.0 / 777, rtol=2e-3)


def test_two_runs_are_bitwise_equal():
    w = synth.scaled(synth.workload(3), seqlens=(4096,), L=3)
    inp = synth.make_qk(w)
    a, la = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, 0.088, orc.LAYER_MAX)
    b, lb = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, 0.088, orc.LAYER_MAX)
    assert (a.view(np.uint32) == b.view(np.uint32)).all() and (la.view(np.uint32) == lb.view(np.uint32)).all()


def test_argument_errors_launch_nothing():
    import torch
    from paper_2502_02789_amd import binding as sp, device as dev
    w = synth.workload(1)
    inp = synth.make_qk(w)
    q = dev.bf16_from_bits(inp["q"])
    ks = [dev.bf16_from_bits(k) for k in inp["k"]]
    cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
    s = dev.Scorer(q, ks, cu, H_kv=w.H_kv, scale=0.125)
    s.scores.fill_(-7.0)
    lib = sp.load_library()
    import ctypes as C

    def status(**changes):
        a = sp.make_score_args(q, ks, cu, s.scores, H_kv=w.H_kv, scale=0.125, workspace=s.workspace)
        for k, v in changes.items():
            setattr(a, k, v)
        return lib.sp_score(C.byref(a), None)

    assert status(d=96) == sp.SP_EINVAL
    assert status(N=17) == sp.SP_EINVAL
    assert status(H_kv=3) == sp.SP_EINVAL
    assert status(layer_reduce=2) == sp.SP_EINVAL
    assert status(d_q=None) == sp.SP_ENULL
    assert status(d_scores=None) == sp.SP_ENULL
    assert status(k_token_stride=w.H_kv * w.d + 4) == sp.SP_EALIGN
    assert status(d_q=q.data_ptr() + 2) == sp.SP_EALIGN
    assert status(workspace_bytes=16) == sp.SP_EWORKSPACE
    assert status(d_workspace=None) == sp.SP_EWORKSPACE
    assert status(rope_theta=5e5) == sp.SP_EUNSUPPORTED
    torch.cuda.synchronize()
    assert (s.scores == -7.0).all()
    assert status() == sp.SP_OK
    torch.cuda.synchronize()
    assert (s.scores > 0).all()


@pytest.mark.parametrize("mode", MODES)
def test_deep_prompt_three_calls_on_one_workspace(mode):
    """Many slabs (the register sets wrap several times, every workgroup takes reducer duties) and
    the same workspace used by consecutive calls: each call must refill what the previous one left."""
    import torch
    from paper_2502_02789_amd import binding as sp_binding, device as dev
    w = synth.scaled(synth.workload(3), seqlens=(8192 + 17,), L=12)
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    want, _ = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, mode)
    q = dev.bf16_from_bits(inp["q"])
    ks = [dev.bf16_from_bits(k) for k in inp["k"]]
    cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
    s = dev.Scorer(q, ks, cu, H_kv=w.H_kv, scale=scale, layer_reduce=mode)
    first = None
    for _ in range(3):
        s.scores.fill_(float("nan"))
        s.run()
        sp_binding.sp_score_check(s.args)
        got = s.scores.cpu().numpy()
        hp.assert_scores_close(got, want, f"{w.name} mode={mode}")
        if first is None:
            first = got
        assert (got.view(np.uint32) == first.view(np.uint32)).all()
