"""GPU parity at the benchmark's own sizes.

Workload 3 (the one bench.py times) runs in full -- every layer, every token -- against
the full fp64 oracle, through the same entry points and launch configuration as the
benchmark.  Workloads 4 and 5 run in full as well (one layer reduction each); their other
cases keep the full token axis, batch structure, head layout and (for 5) the full
128256 x 8192 embedding table with the layer count cut to keep the oracle within seconds.

End-to-end selection (GPU scores -> GPU selection vs oracle scores -> oracle selection):
any chunk kept by one side only must lie within the score tolerance (2e-3 relative) of the
oracle's k-th chunk score.  The stage-isolated check (same fp32 scores on both sides) must
match exactly."""
import math

import numpy as np
import pytest

from oracle import specprefill_oracle as orc
from paper_2502_02789_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _run_whole_path(w, mode, with_table=False, max_seqlen=0):
    import torch
    from paper_2502_02789_amd import binding as sp, device as dev
    inp = synth.make_qk(w, threads=16)
    scale = 1.0 / math.sqrt(w.d)
    ids = synth.make_token_ids(w)
    table = synth.make_embedding(w.vocab, w.embed_dim, w.seed, threads=16) if with_table else None
    cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
    scorer = dev.Scorer(dev.bf16_from_bits(inp["q"]), [dev.bf16_from_bits(k) for k in inp["k"]], cu,
                        H_kv=w.H_kv, scale=scale, layer_reduce=mode, want_lse=True, max_seqlen=max_seqlen)
    scorer.run()
    cap = sp.sp_keep_upper_bound(list(w.seqlens), w.chunk, w.keep_rate)
    sel = dev.Selector(scorer.scores, cu, chunk=w.chunk, pool_window=w.pool_window, keep_rate=w.keep_rate,
                       capacity=cap)
    sel.run()
    gat = dev.Gatherer(sel, token_ids=torch.from_numpy(ids).cuda(),
                       embed=None if table is None else dev.bf16_from_bits(table))
    gat.run()
    torch.cuda.synchronize()

    got = scorer.scores.cpu().numpy()
    want, want_lse = orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], scale, mode)
    err = hp.assert_scores_close(got, want, w.name)
    np.testing.assert_allclose(scorer.lse.cpu().numpy(), want_lse, rtol=0, atol=2e-4)

    kept = sel.kept_idx.cpu().numpy()
    cu_keep = sel.cu_keep.cpu().numpy()
    n = int(cu_keep[-1])
    assert n <= cap
    # stage-isolated: oracle selection on the GPU's own fp32 scores must be identical
    kept_o, cu_keep_o, _, _ = orc.pool_select(got, inp["cu_seqlens"], w.chunk, w.pool_window, w.keep_rate)
    assert cu_keep.tolist() == cu_keep_o.tolist() and (kept[:n] == kept_o).all()
    # end to end: oracle scores -> oracle selection, differences only inside the tolerance window
    swapped = hp.selection_matches(kept[:n], cu_keep, want, inp["cu_seqlens"], w.chunk, w.pool_window,
                                   w.keep_rate, hp.SCORE_RTOL)
    ids_o, pos_o, dec_o, rows_o = orc.gather(kept_o, cu_keep_o, inp["cu_seqlens"], ids, table)
    assert (gat.kept_pos[:n].cpu().numpy() == pos_o).all()
    assert (gat.kept_ids[:n].cpu().numpy() == ids_o).all()
    assert gat.decode_pos.cpu().numpy().tolist() == list(w.seqlens)
    if table is not None:
        assert (dev.bits_from_bf16(gat.out_embed[:n]) == rows_o).all()
    # the planted salient runs must be what gets kept
    sal = inp["salient"]
    keep_mask = np.zeros(w.T, dtype=bool)
    keep_mask[kept[:n]] = True
    print(f"{w.name}: max rel err {err:.2e}, kept {n}, swapped chunks {swapped}, "
          f"salient recall {(keep_mask & sal).sum() / max(1, sal.sum()):.3f}")
    return err


def test_workload_3_full_depth_layer_max():
    _run_whole_path(synth.workload(3), orc.LAYER_MAX)


def test_workload_3_full_depth_layer_mean():
    _run_whole_path(synth.workload(3), orc.LAYER_MEAN)


def test_workload_2_full():
    _run_whole_path(synth.workload(2), orc.LAYER_MAX)


def test_workload_4_ragged_batch_full_tokens():
    _run_whole_path(synth.scaled(synth.workload(4), L=4), orc.LAYER_MAX)


@pytest.mark.parametrize("mode", [orc.LAYER_MAX, orc.LAYER_MEAN])
def test_workload_4_ragged_batch_full_tokens_in_one_pass(mode):
    """The same batch with its longest prompt stated, as bench.py runs it: the single-pass batch kernel
    (eight layers: enough (sequence, layer) units for that kernel to be taken)."""
    w = synth.scaled(synth.workload(4), L=8)
    _run_whole_path(w, mode, max_seqlen=max(w.seqlens))


def test_workload_4_full_depth_in_one_pass():
    """All 32 layers of the 64-prompt workload, exactly what bench.py times on it, against the oracle."""
    w = synth.workload(4)
    _run_whole_path(w, orc.LAYER_MAX, max_seqlen=max(w.seqlens))


def test_workload_4_full_depth_logits_kept_between_two_passes():
    """The same without the longest prompt stated: the MFMA pass that keeps the logits and the pass over those."""
    _run_whole_path(synth.workload(4), orc.LAYER_MEAN)


def test_workload_5_full_depth():
    """All 32 layers of the 128K-token workload (the embedding rows are covered by the four-layer test below)."""
    _run_whole_path(synth.workload(5), orc.LAYER_MAX)


def test_workload_5_full_tokens_and_full_embedding_table():
    _run_whole_path(synth.scaled(synth.workload(5), L=4), orc.LAYER_MAX, with_table=True)


@pytest.mark.parametrize("variant", ["raw", "full", "full_lah"])
def test_paper_variants_as_presets(variant):
    from paper_2502_02789_amd import device as dev
    v = dev.VARIANTS[variant]
    w = synth.scaled(synth.workload(3), seqlens=(3000, 1111), L=3, N=v["n_queries"], chunk=v["chunk"],
                     pool_window=v["pool_window"], keep_rate=0.2, salient_frac=0.02, salient_run=1)
    _run_whole_path(w, orc.LAYER_MAX)


def test_whole_step_replays_from_a_hip_graph():
    """The three calls only enqueue kernels (no allocation, no memset, no synchronisation), so a
    step can be captured once and replayed: three replays, with eager work and synchronisations of
    the program's own in between, must each reproduce the eager result bit for bit."""
    import torch
    from paper_2502_02789_amd import binding as sp, device as dev
    w = synth.scaled(synth.workload(3), seqlens=(9000,), L=4)
    inp = synth.make_qk(w)
    cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
    ids = torch.from_numpy(synth.make_token_ids(w)).cuda()
    scorer = dev.Scorer(dev.bf16_from_bits(inp["q"]), [dev.bf16_from_bits(k) for k in inp["k"]], cu,
                        H_kv=w.H_kv, scale=1.0 / math.sqrt(w.d))
    sel = dev.Selector(scorer.scores, cu, chunk=w.chunk, pool_window=w.pool_window, keep_rate=w.keep_rate)
    gat = dev.Gatherer(sel, token_ids=ids)

    def step():
        scorer.run()
        sel.run()
        gat.run()

    step()                                  # eager: also does the one-time kernel set-up
    torch.cuda.synchronize()
    want = [t.clone() for t in (scorer.scores, sel.kept_idx, sel.cu_keep, gat.kept_pos, gat.kept_ids)]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for replay in range(3):
        for t in (scorer.scores, sel.kept_idx, gat.kept_pos, gat.kept_ids):
            t.fill_(-3)                     # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        sp.sp_score_check(scorer.args)
        n = int(sel.cu_keep[-1])            # (entries beyond the kept count are nobody's to write)
        got = (scorer.scores, sel.kept_idx[:n], sel.cu_keep, gat.kept_pos[:n], gat.kept_ids[:n])
        for a, b in zip(got, (want[0], want[1][:n], want[2], want[3][:n], want[4][:n])):
            assert torch.equal(a, b), f"replay {replay}"
