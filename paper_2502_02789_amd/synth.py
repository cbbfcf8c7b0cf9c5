"""Seeded synthetic inputs shaped like a draft model's stored queries and K cache.

This module only *draws inputs*: Gaussian queries and keys, rotary position
encoding at the true positions (what a serving cache would already hold),
bf16 rounding, and a planted set of "salient" prompt tokens whose keys are
aligned with a look-ahead query.  None of the method's arithmetic (softmax,
aggregation, pooling, selection, gathering) lives here, so both the CPU oracle
tests and the GPU parity tests may draw from it.

Everything is a pure function of (config, seed): each tensor and each layer has
its own counter-based Philox stream, so any layer subset can be re-drawn alone.
bf16 tensors are carried as numpy uint16 bit patterns.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Sequence

import numpy as np

ROPE_THETA = 5.0e5
BASE_SEED = 20250200

# Philox stream ids (second key word = tensor id * 2**20 + layer)
_TID_Q, _TID_K, _TID_SAL, _TID_LEN, _TID_TOK, _TID_EMB = 1, 2, 3, 4, 5, 6


@dataclasses.dataclass(frozen=True)
class Workload:
    """One synthetic scoring workload (shapes follow Llama-3.x draft models)."""
    name: str
    number: int                 # seed offset
    seqlens: tuple              # prompt length M_b of every sequence
    L: int                      # layers
    H: int                      # query heads
    H_kv: int                   # key/value heads
    d: int                      # head dim
    N: int                      # queries per sequence (last token / look-ahead steps)
    chunk: int
    keep_rate: float
    pool_window: int = 13
    salient_frac: float = 0.02
    salient_run: int = 1        # 1 = isolated tokens, 64 = runs of 64 consecutive tokens
    vocab: int = 128256
    embed_dim: int = 0          # 0 = no embedding table in this workload

    @property
    def B(self) -> int:
        return len(self.seqlens)

    @property
    def T(self) -> int:
        return int(sum(self.seqlens))

    @property
    def seed(self) -> int:
        return BASE_SEED + self.number

    def cu_seqlens(self) -> np.ndarray:
        cu = np.zeros(self.B + 1, dtype=np.int32)
        np.cumsum(np.asarray(self.seqlens, dtype=np.int64), out=cu[1:])
        return cu

    def k_bytes(self) -> int:
        return self.T * self.L * self.H_kv * self.d * 2


def _rng(seed: int, tensor_id: int, layer: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, tensor_id * (1 << 20) + layer]))


def _ragged_lengths(seed: int, B: int, lo: int, hi: int) -> tuple:
    return tuple(int(x) for x in _rng(seed, _TID_LEN).integers(lo, hi + 1, size=B))


def workload(number: int) -> Workload:
    """The five benchmark/parity workloads, numbered as in the benchmark definition."""
    if number == 1:
        return Workload("tiny", 1, (1024,), L=2, H=8, H_kv=2, d=64, N=1, chunk=32,
                        keep_rate=0.25, salient_frac=0.02, salient_run=1)
    if number == 2:
        return Workload("1b-8k", 2, (8192,), L=16, H=32, H_kv=8, d=64, N=8, chunk=32,
                        keep_rate=0.1, salient_frac=0.02, salient_run=1)
    if number == 3:
        return Workload("8b-32k", 3, (32768,), L=32, H=32, H_kv=8, d=128, N=8, chunk=32,
                        keep_rate=0.1, salient_frac=0.01, salient_run=64)
    if number == 4:
        return Workload("8b-batch64", 4, _ragged_lengths(BASE_SEED + 4, 64, 1024, 4096),
                        L=32, H=32, H_kv=8, d=128, N=1, chunk=32, keep_rate=0.3,
                        salient_frac=0.01, salient_run=64)
    if number == 5:
        return Workload("8b-128k-gather", 5, (131072,), L=32, H=32, H_kv=8, d=128, N=8,
                        chunk=64, keep_rate=0.05, salient_frac=0.01, salient_run=64,
                        embed_dim=8192)
    raise ValueError(f"unknown workload {number}")


def scaled(w: Workload, **changes) -> Workload:
    """A reduced copy of a workload (fewer layers / shorter prompt) for oracle-sized tests."""
    return dataclasses.replace(w, **changes)


# ----------------------------------------------------------------------------
# bf16 <-> fp32 bit helpers (input formatting only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def rope_rotate(x: np.ndarray, pos: np.ndarray, theta: float = ROPE_THETA) -> np.ndarray:
    """Rotary encoding with the rotate-half pairing (t, t + d/2).

    x: fp32 [..., P, heads, d] with the position axis third from the end; pos: [P].
    """
    d = x.shape[-1]
    half = d // 2
    inv_freq = theta ** (-(np.arange(half, dtype=np.float64) * 2.0) / d)
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]          # [P, half]
    c = np.cos(ang).astype(np.float32)[:, None, :]
    s = np.sin(ang).astype(np.float32)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = lo * c - hi * s
    out[..., half:] = hi * c + lo * s
    return out


def salient_mask(w: Workload) -> np.ndarray:
    """Boolean [T]: the planted salient prompt tokens (same set in every layer)."""
    g = _rng(w.seed, _TID_SAL)
    mask = np.zeros(w.T, dtype=bool)
    cu = w.cu_seqlens()
    for b in range(w.B):
        M = int(cu[b + 1] - cu[b])
        target = max(1, int(round(w.salient_frac * M)))
        if w.salient_run <= 1:
            idx = g.permutation(M)[:target]
            mask[cu[b] + idx] = True
        else:
            run = min(w.salient_run, M)
            n_runs = max(1, int(round(target / run)))
            starts = g.integers(0, M - run + 1, size=n_runs)
            for s0 in starts:
                mask[cu[b] + s0: cu[b] + s0 + run] = True
    return mask


def _draw_layer(w: Workload, layer: int, cu: np.ndarray, sal: np.ndarray):
    """Returns (q bits [B,N,H,d], k bits [T,H_kv,d]) of one layer."""
    G = w.H // w.H_kv
    q_raw = _rng(w.seed, _TID_Q, layer).standard_normal((w.B, w.N, w.H, w.d), dtype=np.float32)
    k_raw = _rng(w.seed, _TID_K, layer).standard_normal((w.T, w.H_kv, w.d), dtype=np.float32)
    q_rot = np.empty_like(q_raw)
    k_rot = np.empty_like(k_raw)
    for b in range(w.B):
        M = int(cu[b + 1] - cu[b])
        q_rot[b] = rope_rotate(q_raw[b], np.arange(M, M + w.N))
        k_rot[cu[b]:cu[b + 1]] = rope_rotate(k_raw[cu[b]:cu[b + 1]], np.arange(M))
    q_bits = f32_to_bf16_bits(q_rot)
    # salient keys: own rotated noise + 3 x (rotated query 0 of the first head of the KV group)
    q0 = bf16_bits_to_f32(q_bits)[:, 0, ::G, :]                          # [B, H_kv, d]
    for b in range(w.B):
        sl = slice(int(cu[b]), int(cu[b + 1]))
        m = sal[sl]
        if m.any():
            seg = k_rot[sl]
            seg[m] = seg[m] + 3.0 * q0[b][None, :, :]
    return q_bits, f32_to_bf16_bits(k_rot)


def make_qk(w: Workload, layers: Optional[Sequence[int]] = None, threads: int = 8) -> Dict[str, object]:
    """Draw the stored queries and the K cache.

    Returns dict with
      q          uint16 [L', B, N, H, d]   (bf16 bits, already rotated)
      k          list of L' arrays uint16 [T, H_kv, d] (token-major, one per layer)
      cu_seqlens int32 [B+1]
      salient    bool [T]
      layers     the layer numbers drawn (L' = len(layers))
    """
    layers = list(range(w.L)) if layers is None else list(layers)
    cu = w.cu_seqlens()
    sal = salient_mask(w)
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        res = list(ex.map(lambda l: _draw_layer(w, l, cu, sal), layers))
    q = np.stack([r[0] for r in res], axis=0)
    k = [r[1] for r in res]
    return {"q": q, "k": k, "cu_seqlens": cu, "salient": sal, "layers": layers}


def make_token_ids(w: Workload) -> np.ndarray:
    return _rng(w.seed, _TID_TOK).integers(0, w.vocab, size=w.T, dtype=np.int32)


def make_embedding(vocab: int, dim: int, seed: int, std: float = 0.02, threads: int = 8,
                   rows_per_block: int = 4096) -> np.ndarray:
    """bf16 bits [vocab, dim] ~ N(0, std), drawn block-wise so blocks are reproducible."""
    out = np.empty((vocab, dim), dtype=np.uint16)
    blocks = list(range(0, vocab, rows_per_block))

    def fill(i0):
        i1 = min(vocab, i0 + rows_per_block)
        x = _rng(seed, _TID_EMB, i0 // rows_per_block).standard_normal((i1 - i0, dim), dtype=np.float32)
        x *= np.float32(std)
        out[i0:i1] = f32_to_bf16_bits(x)

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(fill, blocks))
    return out


def random_scores(seed: int, T: int, ties: bool = False) -> np.ndarray:
    """fp32 importance-like scores for stage-isolated selection tests (positive, heavy-tailed).

    With ties=True values are quantised to a few levels so equal chunk scores are common.
    """
    g = _rng(seed, 7)
    x = np.exp(2.0 * g.standard_normal(T)).astype(np.float32) / np.float32(max(T, 1))
    if ties:
        x = (np.floor(g.random(T) * 4.0) / 4.0 + 0.25).astype(np.float32)
    return x


# ----------------------------------------------------------------------------
# 8-bit K cache (input formatting only): OCP FP8 E4M3 codes with one scale per layer and KV head
# ----------------------------------------------------------------------------
def _e4m3_positive_values() -> np.ndarray:
    """The 127 finite non-negative E4M3 values, code 0x00 .. 0x7E, ascending."""
    code = np.arange(127)
    e, m = code >> 3, code & 7
    return np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))


def quantize_k_fp8(k_bits_layers):
    """bf16 K layers [T, H_kv, d] -> (list of uint8 code arrays, fp32 scales [L, H_kv]).

    What an engine with an 8-bit K cache stores: per layer and KV head one scale = (largest |value|) / 448
    (1 if the head is all zero), each value divided by it (in fp64) and rounded to the nearest E4M3 value,
    ties to the even code, saturating at +-448."""
    vals = _e4m3_positive_values()
    mids = (vals[1:] + vals[:-1]) / 2.0
    codes, scales = [], []
    for k in k_bits_layers:
        x = bf16_bits_to_f32(k).astype(np.float64)
        amax = np.abs(x).max(axis=(0, 2))
        sc = np.where(amax > 0, amax / 448.0, 1.0).astype(np.float32)
        y = np.abs(x) / sc.astype(np.float64)[None, :, None]
        idx = np.searchsorted(mids, y, side="left")             # y <= mids[idx]: value idx is the nearest from below/at the tie
        tie = (idx < len(mids)) & (y == mids[np.minimum(idx, len(mids) - 1)])
        idx = np.where(tie & (idx % 2 == 1), idx + 1, idx)       # a tie goes to the even code
        idx = np.minimum(idx, 126)
        c = idx.astype(np.uint8) | np.where(np.signbit(x), np.uint8(0x80), np.uint8(0)).astype(np.uint8)
        codes.append(np.ascontiguousarray(c))
        scales.append(sc)
    return codes, np.stack(scales).astype(np.float32)
