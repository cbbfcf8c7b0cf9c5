"""GPU parity of the single-pass kernel for batches of short prompts (sp_score with max_seqlen set:
one pass over K, all logits of a sequence kept on chip) against the fp64 oracle, element by
element (Sec. 3.2 equation, Sec. 3.2.2), plus the handling of a broken max_seqlen promise."""
import math

import numpy as np
import pytest

from oracle import specprefill_oracle as orc
from paper_2502_02789_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu

MODES = [orc.LAYER_MAX, orc.LAYER_MEAN]

# 64 sequences: empty, one key, around the 32/64-key tile edges, one wave's worth, all eight waves
# with a ragged last tile, several tiles per wave
LENS_64 = tuple([0, 1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 500, 512, 513, 1029, 1100] + [40 + 7 * i for i in range(48)])


def _lens(seed, B, lo, hi):
    return tuple(int(x) for x in np.random.default_rng(seed).integers(lo, hi + 1, size=B))


def _check(w, inp, mode, max_seqlen, n_valid=None, paged=0, exclusive_device=False):
    scale = 1.0 / math.sqrt(w.d)
    want, want_lse = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, mode, n_valid)
    if paged:
        pools, table = hp.paged_copy(inp["k"], inp["cu_seqlens"], paged, seed=paged)
        got, lse = hp.gpu_score_paged(inp["q"], pools, table, inp["cu_seqlens"], w.H_kv, scale, mode, n_valid=n_valid,
                                      max_seqlen=max_seqlen)
    else:
        got, lse = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, scale, mode, n_valid=n_valid,
                                exclusive_device=exclusive_device, max_seqlen=max_seqlen)
    hp.assert_scores_close(got, want, f"{w.name} mode={mode} max_seqlen={max_seqlen}")
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=2e-4)
    return got


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape", [
    dict(H=8, H_kv=2, N=1, d=128),      # four rows per KV head: the paper's variants without look-ahead on a Llama-shaped draft
    dict(H=8, H_kv=2, N=2, d=128),      # eight rows: two queries
    dict(H=16, H_kv=2, N=1, d=64),      # eight heads per KV head
    dict(H=6, H_kv=2, N=1, d=64),       # three heads, padded to four
    dict(H=10, H_kv=2, N=1, d=128),     # five heads, padded to eight
    dict(H=4, H_kv=4, N=2, d=64),       # one head per KV head (padded to four), two queries
    dict(H=4, H_kv=2, N=1, d=128),      # two heads per KV head (padded to four)
])
def test_batch_of_short_prompts(shape, mode):
    w = synth.scaled(synth.workload(4), seqlens=LENS_64, L=8, salient_frac=0.02, salient_run=1, **shape)
    inp = synth.make_qk(w)
    _check(w, inp, mode, max_seqlen=1100)


@pytest.mark.parametrize("mode", MODES)
def test_longest_sequences_the_registers_hold(mode):
    """8192 keys with four rows per KV head, 4096 with eight: sixteen / eight tiles per wave."""
    w = synth.scaled(synth.workload(4), seqlens=(8192, 8191, 4097) + _lens(5, 125, 1, 90), L=4, H=4, H_kv=1, N=1)
    _check(w, synth.make_qk(w), mode, max_seqlen=8192)
    w = synth.scaled(synth.workload(4), seqlens=(4096, 4033, 2049) + _lens(6, 125, 1, 90), L=4, H=4, H_kv=1, N=2)
    _check(w, synth.make_qk(w), mode, max_seqlen=4096)


def test_valid_query_counts_and_pages():
    w = synth.scaled(synth.workload(4), seqlens=_lens(7, 64, 1, 700), L=8, H=8, H_kv=2, N=2, salient_frac=0.02, salient_run=1)
    inp = synth.make_qk(w)
    nv = np.random.default_rng(8).integers(1, 3, size=64).astype(np.int32)
    for mode in MODES:
        _check(w, inp, mode, max_seqlen=700, n_valid=nv)
        _check(w, inp, mode, max_seqlen=700, n_valid=nv, paged=16)
        _check(w, inp, mode, max_seqlen=700, paged=8)


def test_same_bits_on_every_run_and_with_either_flag():
    w = synth.scaled(synth.workload(4), seqlens=_lens(9, 64, 100, 1500), L=8, H=8, H_kv=2)
    inp = synth.make_qk(w)
    a = _check(w, inp, orc.LAYER_MAX, max_seqlen=1500)
    b = _check(w, inp, orc.LAYER_MAX, max_seqlen=1500, exclusive_device=True)
    assert (a.view(np.uint32) == b.view(np.uint32)).all()


def test_a_sequence_longer_than_promised_gets_nan_scores_and_nothing_else_changes():
    lens = _lens(10, 64, 50, 400)
    w = synth.scaled(synth.workload(4), seqlens=lens[:20] + (8193,) + lens[21:], L=8, H=4, H_kv=1)
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    want, _ = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, orc.LAYER_MAX)
    got, _ = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, scale, orc.LAYER_MAX, max_seqlen=400,
                          exclusive_device=False)
    cu = np.asarray(inp["cu_seqlens"])
    inside = np.zeros(len(got), dtype=bool)
    inside[cu[20]:cu[21]] = True
    assert np.isnan(got[inside]).all()
    hp.assert_scores_close(got[~inside], want[~inside], "the other sequences")
    # the selection answers NaN scores in band
    sel = hp.gpu_pool_select(got, cu, 32, 13, 0.3)
    assert (sel.cu_keep.cpu().numpy()[1:] == -1).all()


def test_without_the_promise_the_two_pass_kernels_give_the_same_scores():
    w = synth.scaled(synth.workload(4), seqlens=_lens(11, 64, 1, 900), L=8, H=8, H_kv=2)
    inp = synth.make_qk(w)
    scale = 1.0 / math.sqrt(w.d)
    a, _ = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, scale, orc.LAYER_MAX, max_seqlen=900)
    b, _ = hp.gpu_score(inp["q"], inp["k"], inp["cu_seqlens"], w.H_kv, scale, orc.LAYER_MAX)
    np.testing.assert_allclose(a, b, rtol=1e-4, atol=0)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("n_keys", [1, 777, 4097, 8192, 8193])
def test_one_prompt_without_look_ahead(n_keys, mode):
    """One sequence: its length is the host's to see, so no promise is needed; the (layer, KV head) slabs are
    dealt out as units of their own (maximum over layers) or layer by layer (mean).  8193 keys are one more
    than the registers hold: the other kernels take over."""
    w = synth.scaled(synth.workload(3), seqlens=(n_keys,), L=4, N=1)
    inp = synth.make_qk(w)
    _check(w, inp, mode, max_seqlen=0, exclusive_device=True)
    _check(w, inp, mode, max_seqlen=0, exclusive_device=False, paged=16 if n_keys == 4097 else 0)


def test_one_prompt_two_queries_and_valid_count():
    w = synth.scaled(synth.workload(3), seqlens=(3000,), L=4, N=2)
    inp = synth.make_qk(w)
    for mode in MODES:
        _check(w, inp, mode, max_seqlen=0, n_valid=np.array([1], dtype=np.int32))
        _check(w, inp, mode, max_seqlen=0)


def test_batch_step_replays_from_a_hip_graph():
    """The batch path only enqueues kernels (ordering, scoring, merge; then selection and gather): captured once
    and replayed three times, with eager work and synchronisations in between, it must reproduce the eager
    result bit for bit."""
    import torch
    from paper_2502_02789_amd import device as dev
    w = synth.scaled(synth.workload(4), seqlens=_lens(12, 64, 1, 1200), L=8, H=8, H_kv=2)
    inp = synth.make_qk(w)
    cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
    scorer = dev.Scorer(dev.bf16_from_bits(inp["q"]), [dev.bf16_from_bits(k) for k in inp["k"]], cu, H_kv=w.H_kv,
                        scale=1.0 / math.sqrt(w.d), max_seqlen=1200, exclusive_device=False)
    sel = dev.Selector(scorer.scores, cu, chunk=w.chunk, pool_window=w.pool_window, keep_rate=w.keep_rate)
    gat = dev.Gatherer(sel)

    def step():
        scorer.run()
        sel.run()
        gat.run()

    step()                                  # eager: also does the one-time kernel set-up
    torch.cuda.synchronize()
    want = [t.clone() for t in (scorer.scores, sel.kept_idx, sel.cu_keep, gat.kept_pos)]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for replay in range(3):
        for t in (scorer.scores, sel.kept_idx, gat.kept_pos):
            t.fill_(-3)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        n = int(sel.cu_keep[-1])
        got = (scorer.scores, sel.kept_idx[:n], sel.cu_keep, gat.kept_pos[:n])
        for a, b in zip(got, (want[0], want[1][:n], want[2], want[3][:n])):
            assert torch.equal(a, b), f"replay {replay}"
