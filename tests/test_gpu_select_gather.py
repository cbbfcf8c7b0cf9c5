"""GPU parity: sp_pool_select and sp_gather (through the C ABI) against the oracle.

Stage-isolated: both sides receive the SAME fp32 score array, so kept indices, positions,
ids and rows must be identical (chunks whose oracle score lies within 1e-6 relative of the
k-th score may swap; with fp64 arithmetic on both sides none are expected to)."""
import numpy as np
import pytest

from oracle import specprefill_oracle as orc
from paper_2502_02789_amd import synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _cu(lens):
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    return cu


CASES = [
    # (lens, chunk, window, keep_rate, ties)
    ((1024,), 32, 13, 0.25, False),
    ((8192,), 32, 13, 0.1, False),
    ((32768,), 32, 13, 0.1, False),
    ((131072,), 64, 13, 0.05, False),
    ((5003,), 32, 13, 0.1, False),          # short last chunk
    ((5003,), 48, 7, 0.3, False),           # chunk that does not divide the wave
    ((4100,), 100, 5, 0.2, False),          # chunk wider than a wave
    ((3000,), 1, 1, 0.1, False),            # the raw variant: token-level top-k, no smoothing
    ((70000,), 1, 1, 0.05, True),           # many equal scores, more chunks than threads
    ((2048,), 16, 3, 0.5, True),
    ((300, 0, 1, 65, 64, 129, 4000), 32, 13, 0.3, False),
    ((300, 0, 1, 65, 64, 129, 4000), 8, 5, 1.0, False),
    ((31,), 32, 13, 0.1, False),            # a single short chunk
]


@pytest.mark.parametrize("lens,chunk,window,rate,ties", CASES)
def test_pool_select_matches_oracle(lens, chunk, window, rate, ties):
    cu = _cu(lens)
    T = int(cu[-1])
    x = synth.random_scores(1234 + T + chunk, T, ties=ties)
    sel = hp.gpu_pool_select(x, cu, chunk, window, rate)
    kept = sel.kept_idx.cpu().numpy()
    cu_keep = sel.cu_keep.cpu().numpy()
    kept_o, cu_keep_o, cs_o, cu_chunks = orc.pool_select(x, cu, chunk, window, rate)
    assert cu_keep.tolist() == cu_keep_o.tolist()
    n = int(cu_keep[-1])
    assert (kept[:n] == kept_o).all()
    assert (kept[n:] == -1).all()                       # untouched beyond the kept count
    cs = sel.chunk_scores.cpu().numpy()[: len(cs_o)]
    np.testing.assert_array_equal(cs, cs_o.astype(np.float32))
    assert hp.selection_matches(kept[:n], cu_keep, x, cu, chunk, window, rate, hp.TIE_RTOL) == 0


def test_all_equal_scores_keep_first_chunks_and_rate_one_keeps_all():
    cu = _cu([4096])
    x = np.full(4096, 0.25, dtype=np.float32)
    sel = hp.gpu_pool_select(x, cu, 32, 13, 0.25)
    n = int(sel.cu_keep[-1])
    assert n == 1024 and sel.kept_idx[:n].cpu().tolist() == list(range(1024))
    sel = hp.gpu_pool_select(synth.random_scores(1, 4096), cu, 32, 13, 1.0)
    assert sel.kept_idx.cpu().tolist() == list(range(4096))


def test_capacity_limits_writes_but_not_counts():
    cu = _cu([4096])
    x = synth.random_scores(5, 4096)
    full = hp.gpu_pool_select(x, cu, 32, 13, 0.25)
    small = hp.gpu_pool_select(x, cu, 32, 13, 0.25, capacity=100)
    assert small.cu_keep.cpu().tolist() == full.cu_keep.cpu().tolist()
    assert (small.kept_idx.cpu()[:100] == full.kept_idx.cpu()[:100]).all()
    from paper_2502_02789_amd import binding as sp
    assert sp.sp_keep_upper_bound([4096], 32, 0.25) == 1024


def test_gather_positions_ids_rows_match_oracle_and_paper_example():
    import torch
    from paper_2502_02789_amd import device as dev
    # the paper's printed example (Sec. 3.2.4): 10 tokens, kept positions 0 1 3 6 7, decoding starts at 10
    scores = np.full(10, 0.01, dtype=np.float32)
    scores[[0, 1, 3, 6, 7]] = [0.9, 0.8, 0.7, 0.6, 0.5]
    sel = hp.gpu_pool_select(scores, _cu([10]), 1, 1, 0.5)
    g = dev.Gatherer(sel)
    g.run()
    torch.cuda.synchronize()
    assert g.kept_pos[:5].cpu().tolist() == [0, 1, 3, 6, 7] and g.decode_pos.cpu().tolist() == [10]

    lens = (300, 0, 1, 65, 64, 129, 4000)
    cu = _cu(lens)
    T = int(cu[-1])
    x = synth.random_scores(77, T)
    sel = hp.gpu_pool_select(x, cu, 32, 13, 0.3)
    rng = np.random.default_rng(3)
    V, D = 1000, 256
    ids = rng.integers(0, V, size=T).astype(np.int32)
    table = rng.integers(0, 65536, size=(V, D)).astype(np.uint16)
    g = dev.Gatherer(sel, token_ids=torch.from_numpy(ids).cuda(), embed=dev.bf16_from_bits(table))
    g.run()
    torch.cuda.synchronize()
    kept_o, cu_keep_o, _, _ = orc.pool_select(x, cu, 32, 13, 0.3)
    ids_o, pos_o, dec_o, rows_o = orc.gather(kept_o, cu_keep_o, cu, ids, table)
    n = len(kept_o)
    assert g.kept_pos[:n].cpu().numpy().tolist() == pos_o.tolist()
    assert g.kept_ids[:n].cpu().numpy().tolist() == ids_o.tolist()
    assert g.decode_pos.cpu().numpy().tolist() == dec_o.tolist() == list(lens)
    assert (dev.bits_from_bf16(g.out_embed[:n]) == rows_o).all()
    assert (g.kept_pos[n:] == -1).all() and (g.out_embed[n:] == 0).all()


def test_select_and_gather_argument_errors():
    import ctypes as C
    import torch
    from paper_2502_02789_amd import binding as sp
    lib = sp.load_library()
    x = synth.random_scores(9, 512)
    sel = hp.gpu_pool_select(x, _cu([512]), 32, 13, 0.25)
    before = sel.kept_idx.clone()

    def status(**changes):
        a = sp.make_pool_select_args(sel.scores, sel.cu, sel.kept_idx, sel.cu_keep, chunk=32, pool_window=13,
                                     keep_rate=0.25, workspace=sel.workspace)
        for k, v in changes.items():
            setattr(a, k, v)
        return lib.sp_pool_select(C.byref(a), None)

    assert status(pool_window=4) == sp.SP_EINVAL
    assert status(chunk=0) == sp.SP_EINVAL
    assert status(keep_rate=0.0) == sp.SP_EINVAL
    assert status(keep_rate=1.5) == sp.SP_EINVAL
    assert status(d_scores=None) == sp.SP_ENULL
    assert status(workspace_bytes=8) == sp.SP_EWORKSPACE
    torch.cuda.synchronize()
    assert (sel.kept_idx == before).all()
    assert status() == sp.SP_OK
    ga = sp.GatherArgs()
    assert lib.sp_gather(C.byref(ga), None) == sp.SP_EINVAL
    assert lib.sp_gather(None, None) == sp.SP_ENULL
    torch.cuda.synchronize()


@pytest.mark.parametrize("T,chunk,rate,ties", [(32768, 32, 0.1, False), (65536, 32, 0.37, True), (1000, 7, 0.5, True)])
def test_single_sequence_fast_path_equals_general_path(T, chunk, rate, ties):
    """One sequence takes the two-launch path; the same tokens followed by an empty sequence take the
    general one.  Both must keep exactly the same tokens."""
    x = synth.random_scores(99 + T, T, ties=ties)
    a = hp.gpu_pool_select(x, _cu([T]), chunk, 13, rate)
    b = hp.gpu_pool_select(x, _cu([T, 0]), chunk, 13, rate)
    na, nb = int(a.cu_keep.cpu()[1]), int(b.cu_keep.cpu()[1])
    assert na == nb == int(b.cu_keep.cpu()[2])
    assert (a.kept_idx.cpu().numpy()[:na] == b.kept_idx.cpu().numpy()[:nb]).all()
    np.testing.assert_array_equal(a.chunk_scores.cpu().numpy()[: (T + chunk - 1) // chunk],
                                  b.chunk_scores.cpu().numpy()[: (T + chunk - 1) // chunk])


@pytest.mark.parametrize("cu", [(0, 700), (0, 300, 300, 1000, 1700)])
def test_nan_scores_are_reported_in_band(cu):
    """A NaN among the scores (the scorer's mark for an expired device-side wait): cu_keep[1..B]
    = -1 and no kept index written, on the single-sequence and on the batched path."""
    rng = np.random.default_rng(3)
    scores = rng.random(cu[-1]).astype(np.float32)
    scores[cu[-1] - 5] = np.nan
    sel = hp.gpu_pool_select(scores, np.array(cu, dtype=np.int32), 32, 5, 0.25)
    assert sel.cu_keep.cpu().tolist() == [0] + [-1] * (len(cu) - 1)
    assert (sel.kept_idx == -1).all()
