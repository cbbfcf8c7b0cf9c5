"""Shared pieces of the GPU parity tests: run the HIP path through the C ABI, run the oracle,
compare under the stated tolerances."""
import math

import numpy as np

from oracle import specprefill_oracle as orc
from paper_2502_02789_amd import synth

SCORE_RTOL = 2e-3          # max relative error of fp32-accumulated scores vs the fp64 oracle
TIE_RTOL = 1e-6            # stage-isolated selection: chunks this close to the k-th score may swap


def gpu_score(q_bits, k_bits_layers, cu, H_kv, scale, mode, n_valid=None, general=False, want_lse=True,
              head_major=False, rope_theta=0.0, q_pos=None, exclusive_device=True, max_seqlen=0):
    import torch
    from paper_2502_02789_amd import binding as sp_binding, device as dev
    q = dev.bf16_from_bits(q_bits)
    if head_major:
        ks = [dev.bf16_from_bits(np.ascontiguousarray(k.transpose(1, 0, 2))).permute(1, 0, 2) for k in k_bits_layers]
    else:
        ks = [dev.bf16_from_bits(k) for k in k_bits_layers]
    cu_d = torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda()
    nv_d = None if n_valid is None else torch.from_numpy(np.asarray(n_valid, dtype=np.int32)).cuda()
    qp_d = None if q_pos is None else torch.from_numpy(np.ascontiguousarray(q_pos, dtype=np.int32)).cuda()
    s = dev.Scorer(q, ks, cu_d, H_kv=H_kv, scale=scale, layer_reduce=mode, n_valid=nv_d, want_lse=want_lse,
                   rope_theta=rope_theta, q_pos=qp_d, exclusive_device=exclusive_device, max_seqlen=max_seqlen)
    s.scores.fill_(float("nan"))
    s.run(general=general)
    sp_binding.sp_score_check(s.args)          # synchronises; raises if a device-side wait expired
    return s.scores.cpu().numpy(), (s.lse.cpu().numpy() if want_lse else None)


def paged_copy(k_bits_layers, cu, page_size, seed, fill=0x7F00):
    """Scatters contiguous [T, H_kv, d] layers into shuffled page pools (with unused pages in
    between); returns (pools, block_table).  Unused rows hold a bit pattern that decodes to a huge
    value, so a kernel that reads a wrong row does not go unnoticed."""
    cu = np.asarray(cu, dtype=np.int64)
    B = len(cu) - 1
    lens = cu[1:] - cu[:-1]
    blocks = [int(-(-m // page_size)) for m in lens]
    bps = max(1, max(blocks))
    n_pages = sum(blocks) + 3
    order = np.random.default_rng(seed).permutation(n_pages)
    table = np.zeros((B, bps), dtype=np.int32)
    nxt = 0
    for b in range(B):
        for j in range(blocks[b]):
            table[b, j] = order[nxt]
            nxt += 1
    pools = []
    for k in k_bits_layers:
        pool = np.full((n_pages, page_size) + k.shape[1:], fill, dtype=k.dtype)   # bf16 1.7e38 (8-bit caches: pass 0x7E = 448)
        for b in range(B):
            for i in range(int(lens[b])):
                pool[table[b, i // page_size], i % page_size] = k[cu[b] + i]
        pools.append(pool)
    return pools, table


def gpu_score_paged(q_bits, pools, table, cu, H_kv, scale, mode, general=False, n_valid=None, max_seqlen=0):
    import torch
    from paper_2502_02789_amd import binding as sp_binding, device as dev
    q = dev.bf16_from_bits(q_bits)
    ks = [dev.bf16_from_bits(p) for p in pools]
    cu_d = torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda()
    tab_d = torch.from_numpy(np.ascontiguousarray(table, dtype=np.int32)).cuda()
    nv_d = None if n_valid is None else torch.from_numpy(np.asarray(n_valid, dtype=np.int32)).cuda()
    s = dev.Scorer(q, ks, cu_d, H_kv=H_kv, scale=scale, layer_reduce=mode, want_lse=True, n_valid=nv_d, block_table=tab_d,
                   page_size=pools[0].shape[1], total_tokens=int(cu[-1]), max_seqlen=max_seqlen)
    s.scores.fill_(float("nan"))
    s.run(general=general)
    sp_binding.sp_score_check(s.args)
    return s.scores.cpu().numpy(), s.lse.cpu().numpy()


def assert_scores_close(got, want, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape
    assert np.isfinite(got).all(), f"{what}: non-finite scores"
    err = np.abs(got - want) / np.maximum(np.abs(want), 1e-300)
    bad = np.abs(got - want) > SCORE_RTOL * np.abs(want) + 1e-30
    assert not bad.any(), f"{what}: max rel err {err.max():.3e} at {int(err.argmax())} ({bad.sum()} over tolerance)"
    return float(err.max())


def gpu_pool_select(scores_f32, cu, chunk, window, keep_rate, capacity=None, want_chunk_scores=True):
    import torch
    from paper_2502_02789_amd import device as dev
    sc = torch.from_numpy(np.ascontiguousarray(scores_f32, dtype=np.float32)).cuda()
    cu_d = torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda()
    sel = dev.Selector(sc, cu_d, chunk=chunk, pool_window=window, keep_rate=keep_rate, capacity=capacity,
                       want_chunk_scores=want_chunk_scores)
    sel.run()
    torch.cuda.synchronize()
    return sel


def selection_matches(kept_gpu, cu_keep_gpu, scores_for_oracle, cu, chunk, window, keep_rate, rtol):
    """Compare a kept-token set with the oracle's.  Chunks may differ only if their oracle chunk
    score lies within rtol (relative) of the oracle's k-th score.  Returns number of swapped chunks."""
    kept_o, cu_keep_o, cs, cu_chunks = orc.pool_select(scores_for_oracle, cu, chunk, window, keep_rate)
    swapped = 0
    for b in range(len(cu) - 1):
        lo, hi = int(cu[b]), int(cu[b + 1])
        g = kept_gpu[int(cu_keep_gpu[b]):int(cu_keep_gpu[b + 1])].astype(np.int64)
        o = kept_o[int(cu_keep_o[b]):int(cu_keep_o[b + 1])]
        assert (np.diff(g) > 0).all(), "kept indices must ascend"
        if len(g) == len(o) and (g == o).all():
            continue
        seg = cs[cu_chunks[b]:cu_chunks[b + 1]]
        k = orc.keep_count(len(seg), keep_rate)
        kth = np.sort(seg)[::-1][k - 1]
        assert ((g >= lo) & (g < hi)).all()
        gc = set(((g - lo) // chunk).tolist())
        oc = set(((o - lo) // chunk).tolist())
        assert len(gc) == len(oc) == k, f"sequence {b}: kept {len(gc)} chunks, oracle {len(oc)}"
        # whole chunks only
        want_tokens = sum(min(chunk, (hi - lo) - j * chunk) for j in gc)
        assert want_tokens == len(g)
        for j in gc ^ oc:
            assert abs(seg[j] - kth) <= rtol * abs(kth), \
                f"sequence {b} chunk {j}: score {seg[j]} vs k-th {kth} outside the tie window"
            swapped += 1
    return swapped


def oracle_scores(inp, w, mode, n_valid=None):
    return orc.token_importance(inp["q"], inp["k"], inp["cu_seqlens"], 1.0 / math.sqrt(w.d), mode, n_valid)
