"""GPU parity of sp_score on a K cache held as 8-bit floats (OCP E4M3 codes with one scale per layer and
KV head) against the fp64 oracle evaluated on the decoded keys (Sec. 3.2 equation, Sec. 3.2.2), element
by element, to the same tolerance as a bf16 cache."""
import math

import numpy as np
import pytest

from oracle import specprefill_oracle as orc
from paper_2502_02789_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu

MODES = [orc.LAYER_MAX, orc.LAYER_MEAN]


def gpu_score_fp8(q_bits, codes, k_scale, cu, H_kv, scale, mode, general=False, n_valid=None, max_seqlen=0,
                  exclusive_device=True, paged=0):
    import torch
    from paper_2502_02789_amd import binding as sp_binding, device as dev
    q = dev.bf16_from_bits(q_bits)
    cu_d = torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda()
    nv_d = None if n_valid is None else torch.from_numpy(np.asarray(n_valid, dtype=np.int32)).cuda()
    sc_d = None if k_scale is None else torch.from_numpy(np.ascontiguousarray(k_scale, dtype=np.float32)).cuda()
    kw = {}
    if paged:
        pools, table = hp.paged_copy(codes, cu, paged, seed=paged, fill=0x7E)
        ks = [torch.from_numpy(p).cuda() for p in pools]
        kw = dict(block_table=torch.from_numpy(np.ascontiguousarray(table, dtype=np.int32)).cuda(), page_size=paged,
                  total_tokens=int(cu[-1]))
    else:
        ks = [torch.from_numpy(np.ascontiguousarray(c)).cuda() for c in codes]
    s = dev.Scorer(q, ks, cu_d, H_kv=H_kv, scale=scale, layer_reduce=mode, n_valid=nv_d, want_lse=True,
                   exclusive_device=exclusive_device, max_seqlen=max_seqlen, k_scale=sc_d, **kw)
    s.scores.fill_(float("nan"))
    s.run(general=general)
    sp_binding.sp_score_check(s.args)
    return s.scores.cpu().numpy(), s.lse.cpu().numpy()


def _check(w, mode, general, n_valid=None, unit_scale=False, **kw):
    inp = synth.make_qk(w)
    codes, k_scale = synth.quantize_k_fp8(inp["k"])
    if unit_scale:
        k_scale = None
    scale = 1.0 / math.sqrt(w.d)
    want, want_lse = orc.token_importance(inp["q"], codes, inp["cu_seqlens"], scale, mode, n_valid,
                                          k_scale=np.ones((w.L, w.H_kv), dtype=np.float32) if unit_scale else k_scale)
    got, lse = gpu_score_fp8(inp["q"], codes, k_scale, inp["cu_seqlens"], w.H_kv, scale, mode, general=general,
                             n_valid=n_valid, **kw)
    hp.assert_scores_close(got, want, f"{w.name} fp8 mode={mode} general={general}")
    # (with the scales left out the decoded keys are up to 448 in size and the log-sum-exps in the thousands:
    # fp32 holds them to 1e-7 relative, hence the relative part)
    np.testing.assert_allclose(lse, want_lse, rtol=1e-6 if unit_scale else 0, atol=2e-4)
    # the quantisation is visible: these are not the bf16 cache's scores
    bf16, _ = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, mode, n_valid)
    if not unit_scale:
        assert np.abs(bf16 - want).max() > 1e-3 * np.abs(want).max()


@pytest.mark.parametrize("general", [False, True])
@pytest.mark.parametrize("mode", MODES)
def test_one_prompt_several_tiles_and_ragged_tail(mode, general):
    _check(synth.scaled(synth.workload(3), seqlens=(1500 + 13,), L=2), mode, general)
    _check(synth.scaled(synth.workload(2), seqlens=(777,), L=3), mode, general)


@pytest.mark.parametrize("general", [False, True])
def test_ragged_batch_valid_query_counts_and_missing_scales(general):
    w = synth.scaled(synth.workload(4), seqlens=(300, 0, 1, 65, 64, 129, 700), L=2, N=2, salient_frac=0.02, salient_run=1)
    for mode in MODES:
        _check(w, mode, general, n_valid=np.array([1, 1, 2, 2, 1, 2, 1], dtype=np.int32))
    _check(w, orc.LAYER_MAX, general, unit_scale=True)


@pytest.mark.parametrize("shape", [dict(H=8, H_kv=8), dict(H=16, H_kv=2), dict(H=6, H_kv=3, N=5), dict(H=5, H_kv=1, N=3)])
def test_other_head_groupings(shape):
    w = synth.scaled(synth.workload(2), seqlens=(517, 90), L=2, **shape)
    for general in (False, True):
        _check(w, orc.LAYER_MAX, general)


@pytest.mark.parametrize("page", [16, 64])
def test_paged_8bit_cache(page):
    w = synth.scaled(synth.workload(4), seqlens=(300, 33, 1000), L=2, salient_frac=0.02, salient_run=1)
    for general in (False, True):
        _check(w, orc.LAYER_MAX, general, paged=page)


def test_argument_rules_of_an_8bit_cache():
    import torch
    from paper_2502_02789_amd import binding as sp, device as dev
    w = synth.scaled(synth.workload(1), seqlens=(128,))
    inp = synth.make_qk(w)
    codes, k_scale = synth.quantize_k_fp8(inp["k"])
    q = dev.bf16_from_bits(inp["q"])
    ks = [torch.from_numpy(c).cuda() for c in codes]
    cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
    s = dev.Scorer(q, ks, cu, H_kv=w.H_kv, scale=0.125, k_scale=torch.from_numpy(k_scale).cuda())
    s.args.rope_theta = 10000.0
    s.args.d_q_pos = s.args.d_cu_seqlens
    with pytest.raises(sp.SpError) as e:
        sp.sp_score(s.args)
    assert e.value.status == sp.SP_EUNSUPPORTED
    s.args.rope_theta = 0.0
    s.args.d_q_pos = None
    s.args.k_token_stride = w.H_kv * w.d + 8          # a multiple of 8 but not of 16
    with pytest.raises(sp.SpError) as e:
        sp.sp_score(s.args)
    assert e.value.status == sp.SP_EALIGN
    s.args.k_token_stride = w.H_kv * w.d
    s.args.k_dtype = 2
    with pytest.raises(sp.SpError) as e:
        sp.sp_score(s.args)
    assert e.value.status in (sp.SP_EINVAL, sp.SP_EWORKSPACE)
    # scales make no sense for a bf16 cache
    b = dev.Scorer(q, [dev.bf16_from_bits(k) for k in inp["k"]], cu, H_kv=w.H_kv, scale=0.125)
    b.args.d_k_scale = s.args.d_k_scale
    with pytest.raises(sp.SpError) as e:
        sp.sp_score(b.args)
    assert e.value.status == sp.SP_EINVAL


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape", [dict(H=8, H_kv=2, N=1, d=128), dict(H=8, H_kv=2, N=2, d=64), dict(H=10, H_kv=2, N=1, d=128)])
def test_batch_of_short_prompts_in_one_pass(shape, mode):
    """The single-pass batch kernel (max_seqlen promised) on an 8-bit cache: tile edges, a sequence of
    several tiles per wave, empty and one-key sequences."""
    lens = (0, 1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 500, 512, 513, 1029, 1100) + tuple(40 + 7 * i for i in range(48))
    w = synth.scaled(synth.workload(4), seqlens=lens, L=8, salient_frac=0.02, salient_run=1, **shape)
    _check(w, mode, False, max_seqlen=1100, exclusive_device=False)
    if shape["d"] == 128:
        _check(w, mode, False, max_seqlen=1100, paged=16)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("n_keys", [5003, 9000 + 13, 16384, 30001, 40000])
def test_one_long_prompt_on_the_single_pass_kernel(n_keys, mode):
    """The 8B shape with the device promised exclusive: sp_score takes the team kernel (more than 8K and up to
    32K keys) or the all-workgroup kernel, which stream the 8-bit keys once."""
    w = synth.scaled(synth.workload(3), seqlens=(n_keys,), L=4 if n_keys < 20000 else 2)
    _check(w, mode, False, n_valid=np.array([5], dtype=np.int32) if n_keys == 16384 else None)


def test_seeded_sweep_of_batch_shapes_bf16_and_8bit_against_the_plain_kernels():
    """Thirty seeded batches that the single-pass batch kernel takes (three to eight heads per KV head, one or two
    queries, both head dims, both layer reductions, contiguous, head-major and paged caches, valid-row counts,
    bf16 and 8-bit keys): sp_score with the longest prompt stated must agree with the plain two-pass kernels on
    the same buffers, which the other tests pin to the oracle."""
    import torch
    from paper_2502_02789_amd import binding as sp_binding, device as dev
    rng = np.random.default_rng(20250208)
    for case in range(30):
        G = int(rng.choice([3, 4, 5, 8]))
        N = int(rng.integers(1, 3)) if G <= 4 else 1
        H_kv = int(rng.choice([1, 2, 4]))
        d = int(rng.choice([64, 128]))
        B = int(rng.integers(2, 70))
        L = max(1, -(-256 // (B * H_kv)) + int(rng.integers(0, 3)))      # enough units for the batch kernel
        lens = tuple(int(x) for x in rng.choice([0, 1, 31, 64, 65, 200, 513, 777, 1500, 2100], size=B))
        if sum(lens) == 0:
            lens = lens[:-1] + (97,)
        mode = MODES[case % 2]
        layout = ("contiguous", "paged", "head_major")[case % 3]
        fp8 = case % 5 in (1, 2)
        w = synth.scaled(synth.workload(4), seqlens=lens, L=L, N=N, H=G * H_kv, H_kv=H_kv, d=d,
                         salient_frac=0.02, salient_run=1)
        inp = synth.make_qk(w)
        cu = inp["cu_seqlens"]
        nv = None if case % 4 == 3 else rng.integers(1, N + 1, size=B).astype(np.int32)
        what = f"case {case}: B={B} G={G} H_kv={H_kv} N={N} d={d} L={L} mode={mode} {layout} fp8={fp8}"
        keys, k_scale = (synth.quantize_k_fp8(inp["k"]) if fp8 else (inp["k"], None))
        kw = {}
        if layout == "paged":
            page = int(rng.choice([16, 32]))
            pools, table = hp.paged_copy(keys, cu, page, seed=case, fill=0x7E if fp8 else 0x7F00)
            ks = [torch.from_numpy(p.view(np.int16) if not fp8 else p).cuda() for p in pools]
            kw = dict(block_table=torch.from_numpy(np.ascontiguousarray(table, dtype=np.int32)).cuda(), page_size=page,
                      total_tokens=int(cu[-1]))
        elif layout == "head_major":
            ks = [torch.from_numpy(np.ascontiguousarray((k.view(np.int16) if not fp8 else k).transpose(1, 0, 2))).cuda().permute(1, 0, 2)
                  for k in keys]
        else:
            ks = [torch.from_numpy(k.view(np.int16) if not fp8 else k).cuda() for k in keys]
        if not fp8:
            ks = [k.view(torch.bfloat16) for k in ks]
        s = dev.Scorer(dev.bf16_from_bits(inp["q"]), ks, torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda(), H_kv=H_kv,
                       scale=1.0 / math.sqrt(d), layer_reduce=mode, want_lse=True, exclusive_device=bool(case & 1),
                       n_valid=None if nv is None else torch.from_numpy(nv).cuda(), max_seqlen=max(lens),
                       k_scale=None if k_scale is None else torch.from_numpy(k_scale).cuda(), **kw)
        s.scores.fill_(float("nan"))
        s.run()
        sp_binding.sp_score_check(s.args)
        a, la = s.scores.cpu().numpy(), s.lse.cpu().numpy()
        s.scores.fill_(float("nan"))
        s.run(general=True)
        torch.cuda.synchronize()
        g, lg = s.scores.cpu().numpy(), s.lse.cpu().numpy()
        np.testing.assert_allclose(a, g, rtol=2e-3, atol=1e-30, err_msg=what)
        np.testing.assert_allclose(la, lg, rtol=1e-6, atol=2e-4, err_msg=what)
