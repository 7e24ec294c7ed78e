"""Seeded synthetic workloads for segment-level attention.

This module only *draws inputs*: bf16 bit patterns for Q, K, V, per-KV-head policy
arrays and decode context lengths.  It contains none of the attention arithmetic, so
the fp64 oracle and the HIP library can both be fed from it without sharing any of
the method's code.

The five workloads mirror the shapes of the paper's long-context experiments
(segment length 4096, carried tail 512-1024, 32 heads of width 128, 16K-128K
tokens; Appendix F "implementation details") with i.i.d. Gaussian values standing in
for real activations.

Everything is a pure function of (workload, seed): values are drawn from numpy's
counter-based Philox generator, one independent key per (tensor, batch index, block of
token rows), so the result does not depend on how the blocks are scheduled over
threads.
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional, Sequence, Tuple

import numpy as np

# Per-KV-head policy bits (which prefix a head's queries may see besides their own
# segment): carried tail of the previous segment, and/or all older rows.
POLICY_SEG = 0
POLICY_TAIL = 1
POLICY_PAST = 2

BASE_SEED = 20260511
_ROWS_PER_BLOCK = 4096
_TENSOR_Q, _TENSOR_K, _TENSOR_V, _TENSOR_AUX, _TENSOR_DOUT = 0, 1, 2, 3, 4


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # 1-based position in the list of benchmark configurations
    batch: int
    seq_len: int               # N (prefill); 0 for the decode workload
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seg_len: int               # S
    tail_len: int              # T
    kv_policy: Tuple[int, ...]  # one policy bitmask per KV head
    outlier_frac: float = 0.0  # fraction of (kv head, channel) pairs of K scaled by 8
    decode: bool = False
    max_context: int = 0       # decode only: upper bound on a sequence's context

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def with_policy(self, kv_policy: Sequence[int]) -> "Workload":
        return dataclasses.replace(self, kv_policy=tuple(int(p) for p in kv_policy))


def _policy(n_kv: int, past_heads: Sequence[int]) -> Tuple[int, ...]:
    return tuple(POLICY_TAIL | POLICY_PAST if h in set(past_heads) else POLICY_TAIL
                 for h in range(n_kv))


C1 = Workload("c1_2k_mha", 1, 1, 2048, 4, 4, 64, 512, 128, _policy(4, (2, 3)))
C2 = Workload("c2_16k_gqa_outliers", 2, 1, 16384, 32, 8, 128, 2048, 512,
              _policy(8, (0, 1)), outlier_frac=0.01)
C3 = Workload("c3_32k_llama3_8b_layer", 3, 1, 32768, 32, 8, 128, 4096, 1024,
              _policy(8, (0, 1, 2, 3)))
C4 = Workload("c4_128k_prefill", 4, 1, 131072, 32, 8, 128, 4096, 1024,
              _policy(8, (0, 1)))
C5 = Workload("c5_decode_b64", 5, 64, 0, 32, 8, 128, 4096, 1024,
              _policy(8, (0, 1)), decode=True, max_context=65536)
WORKLOADS = {w.name: w for w in (C1, C2, C3, C4, C5)}


def interleaved(w: Workload) -> Workload:
    """Same number of PAST heads, spread evenly over the KV heads instead of being the
    lowest indices (the head-grouping ablation, Table 11, contrasts contiguous and
    interleaved groupings; here it only changes load balance, not the FLOP count)."""
    n_past = sum(1 for p in w.kv_policy if p & POLICY_PAST)
    if n_past == 0:
        return w
    step = w.n_kv_heads // n_past
    return w.with_policy(_policy(w.n_kv_heads, [i * step + step // 2 for i in range(n_past)]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def _rng(seed: int, tensor: int, b: int, block: int) -> np.random.Generator:
    key = np.array([np.uint64(seed), (np.uint64(tensor) << np.uint64(48))
                    | (np.uint64(b) << np.uint64(24)) | np.uint64(block)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def _n_threads() -> int:
    return max(1, min(16, len(os.sched_getaffinity(0))))


def normal_bf16(seed: int, tensor: int, batch: int, rows: int, heads: int, dim: int,
                channel_scale: Optional[np.ndarray] = None) -> np.ndarray:
    """bf16 bit patterns of N(0,1) draws, shape [batch, rows, heads, dim] (token-major).

    channel_scale, if given, is a float32 [heads, dim] factor applied before rounding.
    Row block j of batch b always comes from the same Philox key, whatever `rows` is, so
    a shorter tensor is a prefix of a longer one."""
    out = np.empty((batch, rows, heads, dim), dtype=np.uint16)
    jobs = [(b, j) for b in range(batch) for j in range(0, rows, _ROWS_PER_BLOCK)]

    def fill(job):
        b, r0 = job
        n = min(_ROWS_PER_BLOCK, rows - r0)
        x = _rng(seed, tensor, b, r0 // _ROWS_PER_BLOCK).standard_normal(
            (n, heads, dim), dtype=np.float32)
        if channel_scale is not None:
            x = x * channel_scale[None, :, :]
        out[b, r0:r0 + n] = f32_to_bf16_bits(x)

    if len(jobs) == 1:
        fill(jobs[0])
    else:
        with ThreadPoolExecutor(_n_threads()) as ex:
            list(ex.map(fill, jobs))
    return out


def outlier_channel_scale(w: Workload) -> Optional[np.ndarray]:
    """[n_kv_heads, head_dim] float32 factors: round(outlier_frac * Hkv * D) distinct
    (kv head, channel) pairs drawn from the seed are 8, all others 1."""
    if w.outlier_frac <= 0:
        return None
    total = w.n_kv_heads * w.head_dim
    n_out = int(round(w.outlier_frac * total))
    picks = _rng(w.seed, _TENSOR_AUX, 0, 0).choice(total, size=n_out, replace=False)
    s = np.ones(total, dtype=np.float32)
    s[picks] = 8.0
    return s.reshape(w.n_kv_heads, w.head_dim)


def prefill_inputs(w: Workload, seq_len: Optional[int] = None):
    """(q, k, v) bf16 bit patterns for a prefill workload: q [B,N,Hq,D], k,v [B,N,Hkv,D]."""
    n = w.seq_len if seq_len is None else seq_len
    q = normal_bf16(w.seed, _TENSOR_Q, w.batch, n, w.n_q_heads, w.head_dim)
    k = normal_bf16(w.seed, _TENSOR_K, w.batch, n, w.n_kv_heads, w.head_dim,
                    outlier_channel_scale(w))
    v = normal_bf16(w.seed, _TENSOR_V, w.batch, n, w.n_kv_heads, w.head_dim)
    return q, k, v


def grad_inputs(w: Workload, seq_len: Optional[int] = None) -> np.ndarray:
    """Upstream gradient dL/dO for the backward pass: bf16 bit patterns of N(0,1) draws,
    [B,N,Hq,D], from a stream of its own."""
    n = w.seq_len if seq_len is None else seq_len
    return normal_bf16(w.seed, _TENSOR_DOUT, w.batch, n, w.n_q_heads, w.head_dim)


def decode_lengths(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """Per sequence: number of completed segments k_b in 1..max_context/S - 1 and the
    number of tokens c_b in 1..S of the current partial segment *including* the token
    being decoded.  Context length = k_b*S + c_b <= max_context."""
    g = _rng(w.seed, _TENSOR_AUX, 0, 1)
    max_k = w.max_context // w.seg_len - 1
    k_done = g.integers(1, max_k + 1, size=w.batch).astype(np.int64)
    c_fill = g.integers(1, w.seg_len + 1, size=w.batch).astype(np.int64)
    return k_done, c_fill


def decode_inputs(w: Workload, k_done: Optional[np.ndarray] = None,
                  c_fill: Optional[np.ndarray] = None, trailing_rows=None):
    """Decode workload: q [B,Hq,D] bf16 bits for the token being decoded and, per sequence b
    and KV head h, K and V rows [rows, D] of that head's history of n_b = k_b*S + c_b tokens,
    the last row belonging to the token being decoded.  By default the whole history is drawn.
    trailing_rows [B][Hkv], if given, asks for only that many trailing rows of each history:
    input-size bookkeeping for callers whose cache cannot hold (and whose reference zero-fills)
    the older rows of some heads -- the 64-sequence workload is ~3 GB that way instead of ~9 GB.
    Which rows a head may attend to is not decided here."""
    if k_done is None or c_fill is None:
        k_done, c_fill = decode_lengths(w)
    q = normal_bf16(w.seed, _TENSOR_Q, w.batch, 1, w.n_q_heads, w.head_dim)[:, 0]
    jobs = []
    for b in range(w.batch):
        n_b = int(k_done[b]) * w.seg_len + int(c_fill[b])
        for h in range(w.n_kv_heads):
            rows = n_b if trailing_rows is None else min(n_b, int(trailing_rows[b][h]))
            jobs.append((w.seed + 1000 * (b + 1), _TENSOR_K, h, rows, w.head_dim))
            jobs.append((w.seed + 1000 * (b + 1), _TENSOR_V, h, rows, w.head_dim))
    with ThreadPoolExecutor(_n_threads()) as ex:
        res = list(ex.map(lambda a: _head_rows(*a), jobs))
    n_kv = w.n_kv_heads
    ks = [[res[2 * (b * n_kv + h)] for h in range(n_kv)] for b in range(w.batch)]
    vs = [[res[2 * (b * n_kv + h) + 1] for h in range(n_kv)] for b in range(w.batch)]
    return q, ks, vs, k_done, c_fill


def _head_rows(seed: int, tensor: int, head: int, rows: int, dim: int) -> np.ndarray:
    """bf16 bits [rows, dim] for one KV head of one sequence (its own Philox keys)."""
    out = np.empty((rows, dim), dtype=np.uint16)
    for r0 in range(0, rows, _ROWS_PER_BLOCK):
        n = min(_ROWS_PER_BLOCK, rows - r0)
        x = _rng(seed, tensor, head, r0 // _ROWS_PER_BLOCK).standard_normal(
            (n, dim), dtype=np.float32)
        out[r0:r0 + n] = f32_to_bf16_bits(x)
    return out


def small(name: str = "tiny", *, batch=1, seq_len=96, n_q_heads=4, n_kv_heads=2, head_dim=64,
          seg_len=32, tail_len=8, kv_policy: Optional[Sequence[int]] = None,
          index: int = 90) -> Workload:
    """A small workload for tests (same generator, arbitrary shape)."""
    if kv_policy is None:
        kv_policy = [(POLICY_TAIL, POLICY_TAIL | POLICY_PAST, POLICY_SEG, POLICY_PAST)[h % 4]
                     for h in range(n_kv_heads)]
    return Workload(name, index, batch, seq_len, n_q_heads, n_kv_heads, head_dim, seg_len,
                    tail_len, tuple(int(p) for p in kv_policy))
