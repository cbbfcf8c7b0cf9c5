"""CPU oracle for the SpecPrefill token-importance path (arXiv 2502.02789).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the HIP
library is checked against.  Only tests/, the smoke check and the benchmark's
cpu_baseline leg may import it; the product (the C-ABI library and its Python
binding) never does, and it shares no code with them.

Every step is the paper's definition written out in fp64 on the exactly
converted bf16 inputs; numpy's matmul, exp and stable sort are the only library
primitives.  Nothing is blocked, fused or reordered.

Steps and where the paper defines them
  layer_attention      Sec. 3.2 equation  a_ij = Softmax(Q_{M+j} K^T)_i over the M prompt keys
  attention_tensor     Sec. 3.2.2  the [N, L, S, H] score tensor (tiny inputs only)
  aggregate            Sec. 3.2.2  max over H (and L), mean over N
  token_importance     the two above streamed layer by layer (same arithmetic)
  avg_pool             Sec. 3.2.3  1-D average pooling before chunking
  chunk_means          Sec. 3.2.3  contiguous chunks, mean score per chunk
  keep_count           Sec. 4.1    keep rate = ratio of chunks
  select_chunks        Sec. 3.2.3  Top-K chunks
  pool_select          Algorithm 1, chunk_select_from_smoothed_attention
  gather               Sec. 3.2.4  position-id restoration (+ token ids, embedding rows)
  keys_from_pages      Sec. 3.3 / Algorithm 1  keys fetched through the engine's slot mapping (block table)
  fp8_e4m3_bits_to_f64 not in the paper: decoding of a K cache stored as 8-bit floats (OCP FP8, E4M3) with one
                       scale per layer and KV head; the scores are then the paper's on the decoded keys
  rope_rotate_bits     not in the paper: the rotary position encoding a Llama-family draft
                       applies to Q and K before they are cached (needed only when the
                       library is handed an un-rotated cache)

Readings where the paper is silent: softmax over the M
prompt keys only; scale is an argument; pooling window clipped at sequence edges with
the divisor equal to the in-range count; last short chunk averaged over its own
length; k = clamp(ceil(rate * n_chunks - 1e-9), 1, n_chunks); ties go to the lower
index; nothing is force-kept; kept indices ascending.

Parity pins: tests/test_oracle_*.py.  Unpinned: which reading of the layer
reduction / query positions / pooling window the authors' own code uses (the paper
prints no score values) -- "parity unpinned" for those choices only.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

LAYER_MAX = 0    # Sec. 3.2.2 as printed: maximum over heads and layers
LAYER_MEAN = 1   # alternative wording: maximum over heads, mean over layers


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def fp8_e4m3_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact decoding of OCP 8-bit floats, format E4M3 (1 sign, 4 exponent, 3 mantissa bits, bias 7):
    exponent field 0 is subnormal (m/8 * 2^-6), there are no infinities, and the one NaN is
    S.1111.111; the largest finite value is 1.75 * 2^8 = 448."""
    b = np.ascontiguousarray(bits, dtype=np.uint8).astype(np.int64)
    sign = np.where(b >> 7 == 1, -1.0, 1.0)
    e = (b >> 3) & 15
    m = (b & 7).astype(np.float64)
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    sub = (m / 8.0) * 2.0 ** -6
    out = sign * np.where(e == 0, sub, normal)
    return np.where((e == 15) & ((b & 7) == 7), np.nan, out)


def keys_from_fp8(k_codes: np.ndarray, k_scale_layer: np.ndarray) -> np.ndarray:
    """One layer of an 8-bit K cache -> fp64 keys: k_codes uint8 [T, H_kv, d], k_scale_layer fp32 [H_kv];
    key[i, g, :] = scale[g] * decode(code[i, g, :]), the product taken in fp64."""
    scale = np.asarray(k_scale_layer, dtype=np.float32).astype(np.float64)
    return fp8_e4m3_bits_to_f64(k_codes) * scale[None, :, None]


# ----------------------------------------------------------------------------
# a1 + a2: logits and row softmax for one sequence in one layer
# ----------------------------------------------------------------------------
def rope_rotate_bits(x_bits: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position encoding of un-rotated bf16 vectors, result rounded back to bf16.

    x_bits: uint16 bf16 patterns [P, heads, d]; pos: [P] integer positions.  Pair (t, t + d/2)
    is rotated by the angle pos * theta^(-2t/d) (the Llama "rotate-half" convention).  The
    angle is formed in fp64, its cosine and sine are rounded to fp32, the rotation itself is
    done in fp32 and the result is rounded to bf16, nearest-even: this is what a draft model
    running in bf16 with fp32 rotary tables stores in its cache.  Returns uint16 patterns.
    """
    x = (np.asarray(x_bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    d = x.shape[-1]
    half = d // 2
    t = np.arange(half, dtype=np.float64)
    inv_freq = np.power(float(theta), -2.0 * t / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]
    c = np.cos(ang).astype(np.float32)[:, None, :]
    s = np.sin(ang).astype(np.float32)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = lo * c - hi * s
    out[..., half:] = hi * c + lo * s
    u = out.view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def keys_from_pages(pool: np.ndarray, block_table: np.ndarray, cu_seqlens: np.ndarray) -> np.ndarray:
    """Sec. 3.3 / Algorithm 1, the step that fetches the draft's keys through the serving engine's
    slot mapping: `pool` is one layer's page pool [pages, page_size, H_kv, d]; token i of sequence b
    is row i % page_size of page block_table[b, i // page_size].  Returns the layer as [T, H_kv, d]
    rows in cu_seqlens order.  One key at a time, as the definition reads."""
    page_size = pool.shape[1]
    T = int(cu_seqlens[-1])
    out = np.empty((T,) + pool.shape[2:], dtype=pool.dtype)
    for b in range(len(cu_seqlens) - 1):
        for i in range(int(cu_seqlens[b + 1] - cu_seqlens[b])):
            out[int(cu_seqlens[b]) + i] = pool[int(block_table[b, i // page_size]), i % page_size]
    return out


def layer_attention(q: np.ndarray, k: np.ndarray, scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """q fp64 [N, H, d]; k fp64 [M, H_kv, d] -> (a [N, M, H], lse [N, H]).

    Query head h reads KV head h // (H / H_kv).  The softmax runs over the M prompt
    keys of this sequence (Sec. 3.2 equation, 0 <= i < M).
    """
    N, H, d = q.shape
    M, H_kv, _ = k.shape
    G = H // H_kv
    a = np.empty((N, M, H), dtype=np.float64)
    lse = np.empty((N, H), dtype=np.float64)
    for h in range(H):
        kh = k[:, h // G, :]                                   # [M, d]
        s = scale * (q[:, h, :] @ kh.T)                        # [N, M]
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        z = e.sum(axis=1, keepdims=True)
        a[:, :, h] = e / z
        lse[:, h] = (m + np.log(z))[:, 0]
    return a, lse


def attention_tensor(q: np.ndarray, k_layers: Sequence[np.ndarray], scale: float) -> np.ndarray:
    """The paper's score tensor [N, L, S, H] for ONE sequence (tiny inputs only).

    q fp64 [L, N, H, d]; k_layers: L arrays fp64 [S, H_kv, d].
    """
    L = len(k_layers)
    N, H = q.shape[1], q.shape[2]
    S = k_layers[0].shape[0]
    t = np.empty((N, L, S, H), dtype=np.float64)
    for l in range(L):
        t[:, l, :, :], _ = layer_attention(q[l], k_layers[l], scale)
    return t


def aggregate(tensor: np.ndarray, layer_reduce: int = LAYER_MAX) -> np.ndarray:
    """[N, L, S, H] -> importance [S] (Sec. 3.2.2)."""
    over_heads = tensor.max(axis=3)                            # [N, L, S]
    if layer_reduce == LAYER_MAX:
        over_layers = over_heads.max(axis=1)                   # [N, S]
    else:
        over_layers = over_heads.mean(axis=1)
    return over_layers.mean(axis=0)


# ----------------------------------------------------------------------------
# a1..a3 for a ragged batch, streamed over layers (never holds the full tensor)
# ----------------------------------------------------------------------------
def token_importance(q_bits: np.ndarray, k_bits_layers: Sequence[np.ndarray], cu_seqlens: np.ndarray,
                     scale: float, layer_reduce: int = LAYER_MAX,
                     n_valid: Optional[np.ndarray] = None,
                     k_scale: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """q_bits uint16 [L, B, N, H, d]; k_bits_layers: L arrays uint16 [T, H_kv, d] (bf16 bit patterns), or,
    with k_scale (fp32 [L, H_kv]), L arrays uint8 [T, H_kv, d] of 8-bit float codes (keys_from_fp8).

    Returns (scores fp64 [T], lse fp64 [L, B, N, H]).  Only the first n_valid[b]
    queries of sequence b count (EOS validity, Sec. 3.3); their mean is taken.
    Rows of lse belonging to invalid queries are still filled (they are defined).
    """
    L, B, N, H, d = q_bits.shape
    T = int(cu_seqlens[-1])
    scores = np.zeros(T, dtype=np.float64)
    lse = np.zeros((L, B, N, H), dtype=np.float64)
    q = bf16_bits_to_f64(q_bits)
    acc = [None] * B
    for l in range(L):
        k = bf16_bits_to_f64(k_bits_layers[l]) if k_scale is None else keys_from_fp8(k_bits_layers[l], k_scale[l])
        for b in range(B):
            lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
            if hi == lo:
                continue
            a, lse[l, b] = layer_attention(q[l, b], k[lo:hi], scale)
            over_heads = a.max(axis=2)                          # [N, M]
            if acc[b] is None:
                acc[b] = over_heads
            elif layer_reduce == LAYER_MAX:
                acc[b] = np.maximum(acc[b], over_heads)
            else:
                acc[b] = acc[b] + over_heads
    for b in range(B):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        if hi == lo:
            continue
        nv = N if n_valid is None else int(n_valid[b])
        per_query = acc[b] if layer_reduce == LAYER_MAX else acc[b] / L
        scores[lo:hi] = per_query[:nv].sum(axis=0) / nv
    return scores, lse


# ----------------------------------------------------------------------------
# a4: 1-D average pooling, stride 1, same length, window clipped to the sequence
# ----------------------------------------------------------------------------
def avg_pool(scores: np.ndarray, cu_seqlens: np.ndarray, window: int) -> np.ndarray:
    """Mean over [i - r, i + r] intersected with the token's own sequence, r = (window-1)/2.

    The sum is accumulated in index order (offsets -r .. +r) in fp64.
    """
    assert window >= 1 and window % 2 == 1
    r = (window - 1) // 2
    x = np.asarray(scores, dtype=np.float64)
    out = np.zeros_like(x)
    for b in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        M = hi - lo
        if M == 0:
            continue
        seg = x[lo:hi]
        total = np.zeros(M, dtype=np.float64)
        count = np.zeros(M, dtype=np.float64)
        for off in range(-r, r + 1):
            i0, i1 = max(0, -off), min(M, M - off)            # i with 0 <= i + off < M
            if i1 > i0:
                total[i0:i1] += seg[i0 + off:i1 + off]
                count[i0:i1] += 1.0
        out[lo:hi] = total / count
    return out


# ----------------------------------------------------------------------------
# a5: chunk means
# ----------------------------------------------------------------------------
def chunk_means(pooled: np.ndarray, cu_seqlens: np.ndarray, chunk: int) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (chunk scores fp64 [sum_b ceil(M_b/chunk)], cu_chunks int64 [B+1]).

    Chunk j of a sequence covers tokens [j*chunk, min((j+1)*chunk, M)); its score is the
    mean over its actual length, summed in index order.
    """
    B = len(cu_seqlens) - 1
    cu_chunks = np.zeros(B + 1, dtype=np.int64)
    vals: List[float] = []
    for b in range(B):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        M = hi - lo
        n_c = (M + chunk - 1) // chunk
        cu_chunks[b + 1] = cu_chunks[b] + n_c
        for j in range(n_c):
            s0, s1 = lo + j * chunk, min(lo + (j + 1) * chunk, hi)
            tot = 0.0
            for v in pooled[s0:s1]:
                tot += float(v)
            vals.append(tot / (s1 - s0))
    return np.asarray(vals, dtype=np.float64), cu_chunks


# ----------------------------------------------------------------------------
# a6: how many chunks, and which
# ----------------------------------------------------------------------------
def keep_count(n_chunks: int, keep_rate: float) -> int:
    if n_chunks == 0:
        return 0
    k = math.ceil(keep_rate * n_chunks - 1e-9)
    return min(n_chunks, max(1, k))


def select_chunks(chunk_scores: np.ndarray, k: int) -> np.ndarray:
    """Ids of the k largest scores, equal scores resolved to the lower id; ascending ids."""
    order = np.argsort(-np.asarray(chunk_scores, dtype=np.float64), kind="stable")
    return np.sort(order[:k]).astype(np.int64)


# ----------------------------------------------------------------------------
# a4..a7 together
# ----------------------------------------------------------------------------
def pool_select(scores: np.ndarray, cu_seqlens: np.ndarray, chunk: int, window: int,
                keep_rate: float):
    """Returns (kept_idx int64 flat ascending, cu_keep int64 [B+1], chunk_scores fp64, cu_chunks)."""
    pooled = avg_pool(scores, cu_seqlens, window)
    cs, cu_chunks = chunk_means(pooled, cu_seqlens, chunk)
    B = len(cu_seqlens) - 1
    kept: List[np.ndarray] = []
    cu_keep = np.zeros(B + 1, dtype=np.int64)
    for b in range(B):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        seg = cs[cu_chunks[b]:cu_chunks[b + 1]]
        k = keep_count(len(seg), keep_rate)
        n_b = 0
        for j in select_chunks(seg, k):
            s0, s1 = lo + int(j) * chunk, min(lo + (int(j) + 1) * chunk, hi)
            kept.append(np.arange(s0, s1, dtype=np.int64))
            n_b += s1 - s0
        cu_keep[b + 1] = cu_keep[b] + n_b
    kept_idx = np.concatenate(kept) if kept else np.zeros(0, dtype=np.int64)
    return kept_idx, cu_keep, cs, cu_chunks


# ----------------------------------------------------------------------------
# a8: position restoration and gathering
# ----------------------------------------------------------------------------
def gather(kept_idx: np.ndarray, cu_keep: np.ndarray, cu_seqlens: np.ndarray,
           token_ids: Optional[np.ndarray] = None, embed_bits: Optional[np.ndarray] = None):
    """Kept tokens keep their ORIGINAL position inside their own prompt; the first decode
    position of a sequence is its full prompt length (Sec. 3.2.4).

    Returns (kept_ids, kept_pos, decode_pos, rows); kept_ids / rows are None when the
    corresponding input is None.
    """
    B = len(cu_seqlens) - 1
    kept_pos = np.empty(len(kept_idx), dtype=np.int64)
    decode_pos = np.empty(B, dtype=np.int64)
    for b in range(B):
        decode_pos[b] = int(cu_seqlens[b + 1]) - int(cu_seqlens[b])
        for s in range(int(cu_keep[b]), int(cu_keep[b + 1])):
            kept_pos[s] = int(kept_idx[s]) - int(cu_seqlens[b])
    kept_ids = None
    rows = None
    if token_ids is not None:
        kept_ids = np.asarray([int(token_ids[int(i)]) for i in kept_idx], dtype=np.int64)
        if embed_bits is not None:
            V = embed_bits.shape[0]
            assert ((kept_ids >= 0) & (kept_ids < V)).all(), "token id outside the table"
            rows = np.stack([embed_bits[int(t)] for t in kept_ids]) if len(kept_ids) else \
                np.zeros((0, embed_bits.shape[1]), dtype=embed_bits.dtype)
    return kept_ids, kept_pos, decode_pos, rows
