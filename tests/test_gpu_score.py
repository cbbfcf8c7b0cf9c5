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


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("n_valid", [1, 5])
def test_valid_query_count_on_one_long_prompt(n_valid, mode, paged):
    """One prompt, eight KV heads, eight look-ahead rows of which only the first n_valid count
    (Sec. 3.3: look-ahead tokens after an end-of-sequence are not valid): the shape the single-pass
    kernels take, contiguous and behind a block table, against the oracle."""
    w = synth.scaled(synth.workload(3), seqlens=(9000 + 13,), L=3)   # (long enough for either single-pass kernel)
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    nv = np.array([n_valid], dtype=np.int32)
    want, want_lse = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, mode, nv)
    full, _ = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, mode)
    assert np.abs(want - full).max() > 1e-3 * np.abs(full).max()      # the rows left out do matter here
    if paged:
        pools, table = hp.paged_copy(inp["k"], inp["cu_seqlens"], 16, seed=n_valid)
        got, lse = hp.gpu_score_paged(inp["q"], pools, table, inp["cu_seqlens"], w.H_kv, scale, mode, n_valid=nv)
    else:
        got, lse = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, scale, mode, n_valid=nv)
    hp.assert_scores_close(got, want, f"n_valid={n_valid} mode={mode} paged={paged}")
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-4)


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
    assert status(flags=4) == sp.SP_EINVAL                        # an unknown flag bit
    assert status(scale=float("nan")) == sp.SP_EINVAL
    assert status(d_q=None) == sp.SP_ENULL
    assert status(d_scores=None) == sp.SP_ENULL
    assert status(k_token_stride=w.H_kv * w.d + 4) == sp.SP_EALIGN
    assert status(d_q=q.data_ptr() + 2) == sp.SP_EALIGN
    assert status(workspace_bytes=16) == sp.SP_EWORKSPACE
    assert status(d_workspace=None) == sp.SP_EWORKSPACE
    assert status(rope_theta=5e5) == sp.SP_ENULL                  # un-rotated cache without query positions
    assert status(rope_theta=-1.0) == sp.SP_EINVAL
    assert status(d_q_pos=cu.data_ptr()) == sp.SP_EINVAL          # positions given but nothing to rotate
    table = cu.data_ptr()                                          # (never read: the checks come first)
    assert status(d_block_table=table, page_size=12, blocks_per_seq=4) == sp.SP_EINVAL   # not a power of two
    assert status(d_block_table=table, page_size=4, blocks_per_seq=4) == sp.SP_EINVAL    # below eight
    assert status(d_block_table=table, page_size=16, blocks_per_seq=0) == sp.SP_EINVAL
    assert status(d_block_table=table, page_size=16, blocks_per_seq=4, k_page_stride=12) == sp.SP_EALIGN
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


@pytest.mark.parametrize("mode", MODES)
def test_one_long_prompt_without_the_exclusive_device_promise(mode):
    """Without SP_SCORE_EXCLUSIVE_DEVICE the same shape is scored by kernels that never wait for
    another workgroup; same result (to tolerance) as the oracle and as the single-pass kernel."""
    w = synth.scaled(synth.workload(3), seqlens=(5003,), L=3)
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    want, want_lse = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, mode)
    got, lse = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, scale, mode, exclusive_device=False)
    hp.assert_scores_close(got, want, f"shared device, mode={mode}")
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-4)


@pytest.mark.parametrize("tokens", [4096 + 40, 9000])     # the all-workgroup kernel / the team kernel
def test_expired_wait_is_impossible_to_miss(tokens):
    """The single-pass kernels' waits for other workgroups are bounded.  With the bound set to
    zero from the host every wait gives up at once (all kernels still run to their end): the scores
    must then be NaN, sp_score_check must report SP_ETIMEOUT, and selection and gather must hand on
    no keep set.  With the bound restored the same objects give the oracle's result again."""
    import torch
    from paper_2502_02789_amd import binding as sp, device as dev
    w = synth.scaled(synth.workload(3), seqlens=(tokens,), L=3)
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    q = dev.bf16_from_bits(inp["q"])
    ks = [dev.bf16_from_bits(k) for k in inp["k"]]
    cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
    s = dev.Scorer(q, ks, cu, H_kv=w.H_kv, scale=scale)
    sel = dev.Selector(s.scores, cu, chunk=32, pool_window=13, keep_rate=0.1)
    gat = dev.Gatherer(sel, token_ids=torch.zeros(w.T, dtype=torch.int32, device="cuda"))
    before = sp.sp_set_wait_budget(0)
    try:
        assert before > 0 and sp.sp_set_wait_budget(-1) == 0
        s.scores.fill_(1.0)
        sel.kept_idx.fill_(-5)
        s.run()
        sel.run()
        gat.kept_pos.fill_(-5)
        gat.run()
        with pytest.raises(sp.SpError) as e:
            sp.sp_score_check(s.args)
        assert e.value.status == sp.SP_ETIMEOUT
        assert torch.isnan(s.scores).all()
        assert sel.cu_keep.cpu().tolist() == [0, -1]
        assert (sel.kept_idx == -5).all() and (gat.kept_pos == -5).all()
        assert gat.decode_pos.cpu().tolist() == [w.T]
    finally:
        sp.sp_set_wait_budget(before)
    s.run()
    sel.run()
    gat.run()
    sp.sp_score_check(s.args)
    want, _ = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, orc.LAYER_MAX)
    hp.assert_scores_close(s.scores.cpu().numpy(), want, "after the bound was restored")
    assert int(sel.cu_keep[1]) > 0 and (gat.kept_pos[:int(sel.cu_keep[1])] >= 0).all()


@pytest.mark.parametrize("shape", [dict(tokens=9001, L=3), dict(tokens=16500, L=2, H=8, H_kv=8)])
def test_kept_workspace_over_consecutive_calls(shape):
    """SP_SCORE_WORKSPACE_KEPT: a single-pass call leaves its exchange area ready for the next
    one, so from the second call on the kernel that re-initialises it is skipped.  Five calls in a
    row on one workspace (epochs of both parities), a time-out in between (after which the
    workspace starts afresh), the other entry points that write the workspace: every result is
    checked against the oracle, and a kept call's scores equal a fresh call's bit for bit."""
    import torch
    from paper_2502_02789_amd import binding as sp, device as dev
    shape = dict(shape)
    w = synth.scaled(synth.workload(3), seqlens=(shape.pop("tokens"),), **shape)
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    want, _ = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, orc.LAYER_MAX)
    q = dev.bf16_from_bits(inp["q"])
    ks = [dev.bf16_from_bits(k) for k in inp["k"]]
    cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
    s = dev.Scorer(q, ks, cu, H_kv=w.H_kv, scale=scale, keep_workspace=True)
    first = None
    for call in range(5):
        s.scores.fill_(float("nan"))
        s.run()
        assert bool(s.args.flags & sp.SP_SCORE_WORKSPACE_KEPT) == (call > 0)
        s.check()
        got = s.scores.cpu().numpy()
        hp.assert_scores_close(got, want, f"call {call}")
        first = got if first is None else first
        assert np.array_equal(got, first), call
    # a call whose waits give up leaves the workspace in no particular state: the next one starts afresh
    before = sp.sp_set_wait_budget(0)
    try:
        s.run()
        with pytest.raises(sp.SpError):
            s.check()
    finally:
        sp.sp_set_wait_budget(before)
    for call in range(3):
        s.scores.fill_(float("nan"))
        s.run()
        assert bool(s.args.flags & sp.SP_SCORE_WORKSPACE_KEPT) == (call > 0)
        s.check()
        assert np.array_equal(s.scores.cpu().numpy(), first), call
    # the two-pass kernels write the same workspace
    s.run(general=True)
    s.check()
    s.scores.fill_(float("nan"))
    s.run()
    assert not (s.args.flags & sp.SP_SCORE_WORKSPACE_KEPT)
    s.check()
    assert np.array_equal(s.scores.cpu().numpy(), first)


@pytest.mark.parametrize("shape", [
    dict(tokens=9001, H=32, H_kv=8, N=8),      # eight teams, two key tiles per wave and slab, ragged tail
    dict(tokens=16384, H=8, H_kv=8, N=8),      # one query head per KV head, exactly full
    dict(tokens=20011, H=16, H_kv=8, N=3),     # four teams of 64 workgroups, two heads per KV head
    dict(tokens=11000, H=64, H_kv=8, N=4),     # eight heads per KV head
    dict(tokens=10007, H=16, H_kv=4, N=8),     # four KV heads: four teams, one KV head each
    dict(tokens=9500, H=32, H_kv=16, N=2),     # sixteen KV heads: two per team
])
def test_team_kernel_shapes(shape):
    """One prompt of 8K..32K keys, head dim 128, SP_LAYER_MAX: the kernel whose workgroups form teams
    per group of KV heads, in each of its team / tile configurations, against the oracle; twice on
    one workspace, bitwise equal."""
    tokens = shape.pop("tokens")
    w = synth.scaled(synth.workload(3), seqlens=(tokens,), L=3, **shape)
    inp = synth.make_qk(w)
    a = _check(w, inp, orc.LAYER_MAX, general=False)
    got1, lse1 = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, 1.0 / math.sqrt(w.d), orc.LAYER_MAX)
    got2, lse2 = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, 1.0 / math.sqrt(w.d), orc.LAYER_MAX)
    assert np.array_equal(got1, got2) and np.array_equal(lse1, lse2)


@pytest.mark.parametrize("shape", [
    dict(tokens=9001, L=8, H=32, H_kv=8, N=8, n_valid=5),   # eight teams of one layer each, ragged tail, invalid rows
    dict(tokens=20011, L=4, H=16, H_kv=8, N=3),             # four teams, two heads per KV head
    dict(tokens=10007, L=12, H=16, H_kv=4, N=8),            # four KV heads, three layers per team
    dict(tokens=9500, L=4, H=16, H_kv=16, N=2, paged=True), # sixteen KV heads, behind a block table
])
def test_team_kernel_mean_over_layers(shape):
    """SP_LAYER_MEAN on the team kernel: a team owns every TC-th layer (the maximum over a layer's
    heads is then complete inside a workgroup, and the teams' sums over their layers add up),
    against the oracle; twice on one workspace, bitwise equal."""
    shape = dict(shape)
    tokens, n_valid, paged = shape.pop("tokens"), shape.pop("n_valid", None), shape.pop("paged", False)
    w = synth.scaled(synth.workload(3), seqlens=(tokens,), **shape)
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    nv = None if n_valid is None else np.array([n_valid], dtype=np.int32)
    want, want_lse = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, orc.LAYER_MEAN, nv)
    runs = []
    for _ in range(2):
        if paged:
            pools, table = hp.paged_copy(inp["k"], inp["cu_seqlens"], 16, seed=3)
            runs.append(hp.gpu_score_paged(inp["q"], pools, table, inp["cu_seqlens"], w.H_kv, scale, orc.LAYER_MEAN, n_valid=nv))
        else:
            runs.append(hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, scale, orc.LAYER_MEAN, n_valid=nv))
    hp.assert_scores_close(runs[0][0], want, f"team kernel, mean over layers {shape}")
    np.testing.assert_allclose(runs[0][1], want_lse, rtol=0, atol=2e-4)
    assert np.array_equal(runs[0][0], runs[1][0]) and np.array_equal(runs[0][1], runs[1][1])


def _raw_inputs(seed, seqlens, L, H, H_kv, d, N):
    """Un-rotated bf16 Q [L,B,N,H,d] and per-layer K [T,H_kv,d], plus query positions [B,N]."""
    rng = np.random.default_rng(seed)
    B, T = len(seqlens), int(sum(seqlens))
    q = synth.f32_to_bf16_bits(rng.standard_normal((L, B, N, H, d)).astype(np.float32))
    k = [synth.f32_to_bf16_bits(rng.standard_normal((T, H_kv, d)).astype(np.float32)) for _ in range(L)]
    cu = np.zeros(B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(seqlens)
    q_pos = np.array([[m + n for n in range(N)] for m in seqlens], dtype=np.int32)
    return q, k, cu, q_pos


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape", [((700, 33, 0, 1290), 2, 8, 2, 64, 3), ((2100,), 2, 32, 8, 128, 8)])
def test_unrotated_cache_is_rotated_by_the_library(shape, mode):
    """rope_theta > 0: raw Q and K in, same scores as the oracle gets after rotating them itself."""
    seqlens, L, H, H_kv, d, N = shape
    theta = 5e5
    q, k, cu, q_pos = _raw_inputs(11, seqlens, L, H, H_kv, d, N)
    q_rot = np.stack([np.stack([orc.rope_rotate_bits(q[l, b], q_pos[b], theta) for b in range(len(seqlens))])
                      for l in range(L)])
    k_rot = []
    for l in range(L):
        kr = np.empty_like(k[l])
        for b in range(len(seqlens)):
            lo, hi = int(cu[b]), int(cu[b + 1])
            kr[lo:hi] = orc.rope_rotate_bits(k[l][lo:hi], np.arange(hi - lo), theta)
        k_rot.append(kr)
    scale = 1.0 / math.sqrt(d)
    want, want_lse = orc.token_importance(q_rot, k_rot, cu, scale, mode)
    got, lse = hp.gpu_score(q, k, cu, H_kv, scale, mode, rope_theta=theta, q_pos=q_pos)
    hp.assert_scores_close(got, want, f"raw cache {shape} mode={mode}")
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-3)


def test_rotation_by_position_zero_changes_nothing():
    """All positions zero is the identity rotation: bit-identical to the already-rotated path."""
    q, k, cu, _ = _raw_inputs(12, (1,), 2, 8, 2, 64, 1)      # one key at position 0, one query at position 0
    zero_pos = np.zeros((1, 1), dtype=np.int32)
    for general in (True, False):   # the plain kernels, and the MFMA kernels sp_score picks for this shape
        a, la = hp.gpu_score(q, k, cu, 2, 0.125, orc.LAYER_MAX, general=general)
        b, lb = hp.gpu_score(q, k, cu, 2, 0.125, orc.LAYER_MAX, general=general, rope_theta=1e4, q_pos=zero_pos)
        assert (a.view(np.uint32) == b.view(np.uint32)).all() and (la.view(np.uint32) == lb.view(np.uint32)).all()


@pytest.mark.parametrize("shape", [
    ((300, 1, 97, 64, 65), 3, 8, 8, 128, 1),     # one row per KV head: logits kept between the passes, head dim 128
    ((1500,), 5, 12, 4, 64, 2),                   # three heads per KV head (padded to four), several layer groups
    ((40, 2000), 2, 32, 8, 128, 8),               # thirty-two rows per KV head, both layer modes below
])
@pytest.mark.parametrize("mode", MODES)
def test_mfma_kernels_rotate_like_the_plain_kernels(shape, mode):
    """rope_theta > 0 on the MFMA kernels (keys turned in registers on their way to the matrix
    cores) against the plain kernels, which turn them one row per lane: same rounding chain, so
    the two agree as closely as they do on an already-rotated cache; and against the oracle."""
    seqlens, L, H, H_kv, d, N = shape
    theta = 5e5
    q, k, cu, q_pos = _raw_inputs(13, seqlens, L, H, H_kv, d, N)
    scale = 1.0 / math.sqrt(d)
    fast, lse_fast = hp.gpu_score(q, k, cu, H_kv, scale, mode, rope_theta=theta, q_pos=q_pos, exclusive_device=False)
    plain, lse_plain = hp.gpu_score(q, k, cu, H_kv, scale, mode, rope_theta=theta, q_pos=q_pos, general=True)
    hp.assert_scores_close(fast, plain.astype(np.float64), f"MFMA vs plain kernels, raw cache {shape} mode={mode}")
    np.testing.assert_allclose(lse_fast, lse_plain, rtol=0, atol=2e-4)
    q_rot = np.stack([np.stack([orc.rope_rotate_bits(q[l, b], q_pos[b], theta) for b in range(len(seqlens))])
                      for l in range(L)])
    k_rot = []
    for l in range(L):
        kr = np.empty_like(k[l])
        for b in range(len(seqlens)):
            lo, hi = int(cu[b]), int(cu[b + 1])
            kr[lo:hi] = orc.rope_rotate_bits(k[l][lo:hi], np.arange(hi - lo), theta)
        k_rot.append(kr)
    want, _ = orc.token_importance(q_rot, k_rot, cu, scale, mode)
    hp.assert_scores_close(fast, want, f"MFMA kernels, raw cache {shape} mode={mode}")
    # and the canonical path on the oracle-rotated cache gives the same scores bit for bit:
    # rotating inside the kernel is the same as reading a rotated cache
    canon, _ = hp.gpu_score(q_rot, k_rot, cu, H_kv, scale, mode, exclusive_device=False)
    assert np.array_equal(fast.view(np.uint32), canon.view(np.uint32))


# The ragged-batch MFMA kernels (what sp_score picks for B > 1): every tile-boundary case of
# the 64-key wave tiles and of their two 32-key halves, several layer groups, both modes.
@pytest.mark.parametrize("shape", [
    dict(H=32, H_kv=8, d=128, N=1, L=5),
    dict(H=32, H_kv=8, d=128, N=8, L=3),
    dict(H=24, H_kv=3, d=64, N=4, L=4),
    dict(H=5, H_kv=5, d=64, N=16, L=2),
    dict(H=3, H_kv=3, d=64, N=3, L=3),     # three query rows per KV head: logits kept between the passes
    dict(H=4, H_kv=2, d=128, N=2, L=2),    # four rows from two queries x two heads
    dict(H=32, H_kv=8, d=128, N=2, L=3),   # eight rows (one look-ahead step): logits kept as two 16-byte units
    dict(H=16, H_kv=2, d=64, N=1, L=2),    # eight heads per KV head
    dict(H=6, H_kv=3, d=64, N=3, L=2),     # six rows: the second unit is partly padding
])
def test_ragged_batch_tile_boundaries(shape):
    lens = (1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 0, 700)
    w = synth.scaled(synth.workload(4), seqlens=lens, salient_frac=0.02, salient_run=1, **shape)
    inp = synth.make_qk(w)
    nv = np.array([1 + (i % shape["N"]) for i in range(len(lens))], dtype=np.int32)
    for mode in MODES:
        _check(w, inp, mode, general=False, n_valid=nv)


def test_ragged_batch_paths_agree_and_repeat_bitwise():
    w = synth.scaled(synth.workload(4), seqlens=(1500, 77, 2049, 640), L=4)
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    for mode in MODES:
        a, la = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, scale, mode)
        b, lb = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, scale, mode)
        g, lg = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, scale, mode, general=True)
        assert np.array_equal(a, b) and np.array_equal(la, lb)
        np.testing.assert_allclose(a, g, rtol=2e-3, atol=1e-12)
        np.testing.assert_allclose(la, lg, rtol=0, atol=2e-4)


def test_maximum_depth_on_every_path():
    """L = SP_MAX_LAYERS: one long-ish prompt (single-pass kernel), a ragged batch with look-ahead
    queries (two MFMA passes), one without (logits kept between the passes), and the plain kernels."""
    for lens, n in (((2000,), 8), ((700, 150, 1), 8), ((700, 150, 1), 1)):
        w = synth.scaled(synth.workload(2), seqlens=lens, L=128, N=n, salient_frac=0.02, salient_run=1)
        inp = synth.make_qk(w)
        for mode in MODES:
            _check(w, inp, mode, general=False)
        _check(w, inp, orc.LAYER_MAX, general=True)


@pytest.mark.parametrize("n_queries", [1, 8])
def test_head_major_k_layout_ragged_batch(n_queries):
    """[H_kv, T, d] caches through the ragged-batch kernels (both of their second passes)."""
    w = synth.scaled(synth.workload(3), seqlens=(333, 64, 1000), L=3, N=n_queries)
    inp = synth.make_qk(w)
    for mode in MODES:
        _check(w, inp, mode, general=False, head_major=True)


@pytest.mark.parametrize("shape", [
    dict(H=14, H_kv=2, d=64, N=4),    # seven heads per KV head (padded to eight columns per query)
    dict(H=12, H_kv=2, d=128, N=1),   # six
    dict(H=9, H_kv=3, d=64, N=1),     # three: logits kept between the passes, one padding column
    dict(H=5, H_kv=1, d=128, N=2),    # five
])
def test_group_sizes_that_are_not_powers_of_two(shape):
    w = synth.scaled(synth.workload(2), seqlens=(130, 517, 64), L=3, salient_frac=0.02, salient_run=1, **shape)
    inp = synth.make_qk(w)
    for mode in MODES:
        a = _check(w, inp, mode, general=False)
    _check(w, inp, orc.LAYER_MAX, general=True)


@pytest.mark.parametrize("page_size", [8, 16, 64])
@pytest.mark.parametrize("n_queries", [1, 8])
def test_paged_cache(page_size, n_queries):
    """Keys fetched through a block table (shuffled pages, partly filled last pages) give what the
    same keys give when they lie in sequence order; oracle: gather the pages, then as always."""
    w = synth.scaled(synth.workload(3), seqlens=(333, 64, 1, 0, 1000), L=3, N=n_queries, salient_frac=0.02,
                     salient_run=1)
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    pools, table = hp.paged_copy(inp["k"], inp["cu_seqlens"], page_size, seed=page_size)
    k_back = [orc.keys_from_pages(p, table, inp["cu_seqlens"]) for p in pools]
    for mode in MODES:
        want, want_lse = orc.token_importance(inp["q"], k_back, inp["cu_seqlens"], scale, mode)
        for general in (False, True):
            got, lse = hp.gpu_score_paged(inp["q"], pools, table, inp["cu_seqlens"], w.H_kv, scale, mode, general)
            hp.assert_scores_close(got, want, f"paged {page_size} mode={mode} general={general}")
            np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-4)


@pytest.mark.parametrize("page_size", [8, 16, 128])
def test_paged_single_prompt(page_size):
    """One long prompt behind a block table: the single-pass kernel reads the table itself.
    Ragged tail, several key tiles per workgroup."""
    w = synth.scaled(synth.workload(3), seqlens=(16500,), L=3)
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    pools, table = hp.paged_copy(inp["k"], inp["cu_seqlens"], page_size, seed=3)
    for mode in MODES:
        want, want_lse = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, mode)
        got, lse = hp.gpu_score_paged(inp["q"], pools, table, inp["cu_seqlens"], w.H_kv, scale, mode)
        hp.assert_scores_close(got, want, f"paged single prompt, page {page_size}, mode {mode}")
        np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-4)
        again, _ = hp.gpu_score_paged(inp["q"], pools, table, inp["cu_seqlens"], w.H_kv, scale, mode)
        assert np.array_equal(got, again)


def test_seeded_shape_sweep_fast_paths_agree_with_the_plain_kernels():
    """Forty seeded shapes (group sizes 1..8, ragged batches with empty and one-key sequences,
    both head dims, contiguous and paged caches, both modes, valid-row counts): whatever kernels sp_score picks must
    agree with the plain two-pass kernels, which the other tests pin to the oracle."""
    rng = np.random.default_rng(20250207)
    for case in range(40):
        G = int(rng.integers(1, 9))
        Gp = 1 if G == 1 else 2 if G == 2 else 4 if G <= 4 else 8
        H_kv = int(rng.choice([1, 2, 3, 8]))
        N = int(rng.integers(1, min(16, 32 // Gp) + 1))
        d = int(rng.choice([64, 128]))
        L = int(rng.integers(1, 5))
        B = int(rng.integers(1, 6))
        lens = tuple(int(x) for x in rng.choice([0, 1, 31, 64, 65, 200, 777, 1500], size=B))
        if sum(lens) == 0:
            lens = lens[:-1] + (97,)
        mode = MODES[case % 2]
        paged = case % 3 == 0
        w = synth.scaled(synth.workload(2), seqlens=lens, L=L, N=N, H=G * H_kv, H_kv=H_kv, d=d,
                         salient_frac=0.02, salient_run=1)
        inp = synth.make_qk(w)
        scale = 1.0 / math.sqrt(d)
        nv = None if case % 4 == 3 else rng.integers(1, N + 1, size=B).astype(np.int32)   # valid look-ahead rows
        what = f"case {case}: lens={lens} G={G} H_kv={H_kv} N={N} d={d} L={L} mode={mode} paged={paged} n_valid={nv}"
        if paged:
            pools, table = hp.paged_copy(inp["k"], inp["cu_seqlens"], int(rng.choice([8, 16, 32])), seed=case)
            a, la = hp.gpu_score_paged(inp["q"], pools, table, inp["cu_seqlens"], H_kv, scale, mode, n_valid=nv)
            g, lg = hp.gpu_score_paged(inp["q"], pools, table, inp["cu_seqlens"], H_kv, scale, mode, general=True,
                                       n_valid=nv)
        else:
            a, la = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], H_kv, scale, mode, n_valid=nv)
            g, lg = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], H_kv, scale, mode, general=True, n_valid=nv)
        np.testing.assert_allclose(a, g, rtol=2e-3, atol=1e-30, err_msg=what)
        np.testing.assert_allclose(la, lg, rtol=0, atol=2e-4, err_msg=what)
