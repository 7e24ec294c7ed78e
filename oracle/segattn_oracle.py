"""fp64 CPU oracle for segment-level causal attention.  TEST INFRASTRUCTURE ONLY.

This file is the plain definition of what the HIP library must compute, written from
the paper and kept deliberately slow and obvious.  It is imported only by the tests,
by the smoke check and by the benchmark's CPU-baseline leg; the product path never
calls it, and it shares no code with the GPU path (it does not import the package).

What it computes (Appendix C, "Attention Contexts for Local and Long-Range Heads"):

* Eq. 12: Attn(Q,K,V) = softmax(Q K^T / sqrt(d) + M) V, where the mask M lets a
  segment query see every prefix row and the rows of its own segment up to itself.
* Eq. 13: which prefix a head sees.  A *local* head sees the carried KV tail, i.e. the
  last M key/value rows of the previous segment (Sec. 3.4, "Local Continuity
  Channel").  A *long-range* head in a long-range layer sees forward-only past KV
  (Sec. 3.4, "Long-Range Channel"); elsewhere it sees its own segment only.
* First segment: C_0 = R_0 = empty (Sec. 3.1, "Operational interpretation").

Readings taken where the paper is silent (each is repeated in the design notes):

* The policy is a bit mask per KV head, TAIL = 1, PAST = 2; a head with both bits sees
  the *union of positions* (a key is never counted twice).  The query heads of a GQA
  group inherit the policy of their KV head, which is query head // group size.
* "Past" is every position before the current segment (minus `evicted` oldest ones) by
  default.  With `retrieved` given it is the paper's own form (Eq. 13, second case;
  Appendix D "Output"): the R pool rows an index list names, as a set of distinct
  positions before the segment.  How the list is chosen (top-k scoring, anchors, window
  expansion of Appendix D) is not part of this file.
* The tail is the last min(T, length of the previous segment) rows of the previous
  segment only; T <= S is required.  Segments start at multiples of S; only the last
  one may be short.
* LSE is the natural log of sum_j exp(scale * q.k_j) over the visible keys.

Everything is written over absolute token positions with an explicit boolean mask per
query row, dense scores over all N keys, -inf where masked, and a plain softmax.
Inputs are bf16 bit patterns (uint16) or floats; bf16 is widened exactly to fp64.
retrieve_indices() is the retrieval operator of Appendix D under stated readings of its
unstated parameters: PARITY UNPINNED against the paper (it prints no values, k, anchor count,
window or fallback); its pins check the reading against its own literal description.
rope_rotate() / attend_reindexed() are the RoPE re-indexing of Appendix E written literally.
attend_backward() is the gradient of the same definition (dQ, dK, dV), with gradient stopped
where the paper stops it (past rows are forward-only; the carried tail is differentiable).
All pins for this file live in tests/test_oracle_*.py; no function here is unpinned.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import numpy as np

POLICY_SEG = 0
POLICY_TAIL = 1
POLICY_PAST = 2


def widen(x: np.ndarray) -> np.ndarray:
    """Exact float64 value of a uint16 bf16 bit pattern (or of any float array)."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


def visible_mask(p: int, n: int, seg_len: int, tail_len: int, policy: int,
                 evicted: int = 0, retrieved=None) -> np.ndarray:
    """Boolean [n]: which key positions query position p may attend to (Eq. 12 mask,
    Eq. 13 context).  Segment i = p // S starts at s = i*S.  `retrieved`, if not None, is
    the retrieved prefix of p's segment for a PAST head: distinct positions < s."""
    if not (0 <= tail_len <= seg_len):
        raise ValueError("need 0 <= tail_len <= seg_len")
    if not (0 <= p < n):
        raise ValueError("query position outside the sequence")
    s = (p // seg_len) * seg_len
    j = np.arange(n)
    vis = (j >= s) & (j <= p)                      # own segment, causal (all cases of Eq. 13)
    if policy & POLICY_TAIL:                       # carried tail: last T rows of segment i-1
        vis |= (j >= max(0, s - tail_len)) & (j < s)
    if policy & POLICY_PAST:
        if retrieved is None:                      # forward-only past: every earlier row kept
            vis |= (j >= evicted) & (j < s)
        else:                                      # forward-only past: the R retrieved rows
            idx = np.asarray(retrieved, dtype=np.int64).reshape(-1)
            if idx.size and (idx.min() < evicted or idx.max() >= s):
                raise ValueError("retrieved position outside the pool of this segment")
            if np.unique(idx).size != idx.size:
                raise ValueError("retrieved positions must be distinct")
            vis[idx] = True
    return vis


def _rows_arg(rows, n):
    if rows is None:
        return np.arange(n, dtype=np.int64)
    rows = np.asarray(rows, dtype=np.int64).reshape(-1)
    if rows.size and (rows.min() < 0 or rows.max() >= n):
        raise ValueError("row outside the sequence")
    return rows


def attend(q, k, v, *, seg_len: int, tail_len: int, kv_policy: Sequence[int],
           scale: Optional[float] = None, rows=None, evicted: Optional[Sequence[int]] = None,
           return_probs: bool = False, max_block_bytes: int = 1 << 28, retrieved=None):
    """Segment-level attention for the query positions `rows` (default: all).

    q [B,N,Hq,D]; k, v [B,N,Hkv,D]; returns O [B,R,Hq,D] and LSE [B,Hq,R] in float64
    (and the probabilities [B,Hq,R,N] if return_probs).  evicted[h] = number of oldest
    rows KV head h no longer holds (only PAST visibility is affected).  retrieved, if
    given, maps (b, kv head, segment index) to the positions of that segment's retrieved
    prefix; PAST heads then see those rows instead of the whole history (a missing key
    means an empty prefix)."""
    q, k, v = widen(q), widen(k), widen(v)
    B, N, Hq, D = q.shape
    Hkv = k.shape[2]
    if k.shape != (B, N, Hkv, D) or v.shape != k.shape:
        raise ValueError("shape mismatch")
    if Hq % Hkv or len(kv_policy) != Hkv:
        raise ValueError("bad head configuration")
    g = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    rows = _rows_arg(rows, N)
    R = rows.size
    ev = [0] * Hkv if evicted is None else [int(e) for e in evicted]
    out = np.zeros((B, R, Hq, D))
    lse = np.zeros((B, Hq, R))
    probs = np.zeros((B, Hq, R, N)) if return_probs else None
    step = max(1, int(max_block_bytes // (8 * max(N, 1))))
    for kvh in range(Hkv):
        pol = int(kv_policy[kvh])
        for r0 in range(0, R, step):
            rr = rows[r0:r0 + step]
            def mask_for(b):
                if not rr.size:
                    return np.zeros((0, N), dtype=bool)
                if retrieved is None:
                    return np.stack([visible_mask(int(p), N, seg_len, tail_len, pol, ev[kvh]) for p in rr])
                return np.stack([visible_mask(int(p), N, seg_len, tail_len, pol, ev[kvh],
                                              retrieved.get((b, kvh, int(p) // seg_len), ()))
                                 for p in rr])
            mask = mask_for(0)
            for b in range(B):
                if retrieved is not None and b > 0:
                    mask = mask_for(b)
                kb, vb = k[b, :, kvh, :], v[b, :, kvh, :]
                for h in range(kvh * g, (kvh + 1) * g):
                    z = (q[b, rr, h, :] @ kb.T) * scale          # dense scores, all N keys
                    z = np.where(mask, z, -np.inf)               # + M of Eq. 12
                    zmax = z.max(axis=1, keepdims=True)
                    e = np.exp(z - zmax)
                    denom = e.sum(axis=1, keepdims=True)
                    pr = e / denom                               # softmax
                    out[b, r0:r0 + rr.size, h, :] = pr @ vb
                    lse[b, h, r0:r0 + rr.size] = (zmax + np.log(denom))[:, 0]
                    if return_probs:
                        probs[b, h, r0:r0 + rr.size, :] = pr
    if return_probs:
        return out, lse, probs
    return out, lse


def attend_packed(q, k, v, cu_seqlens, **kw):
    """A ragged batch packed without padding: q [total,Hq,D], k, v [total,Hkv,D]; sequence b is
    rows cu_seqlens[b] .. cu_seqlens[b+1]-1 and is processed on its own (its segments start at
    multiples of S counted from its first row; nothing crosses a sequence boundary -- the
    sequences of a batch are independent samples in Eq. 12-13).  Returns O [total,Hq,D] and
    LSE [Hq,total]; keyword arguments as for attend()."""
    total, Hq, D = q.shape
    out, lse = np.zeros((total, Hq, D)), np.zeros((Hq, total))
    for b in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        if hi > lo:
            o, l = attend(q[None, lo:hi], k[None, lo:hi], v[None, lo:hi], **kw)
            out[lo:hi], lse[:, lo:hi] = o[0], l[0]
    return out, lse


def decode_attend(q, k_ctx, v_ctx, *, seg_len: int, tail_len: int, kv_policy: Sequence[int],
                  scale: Optional[float] = None, evicted: Optional[Sequence[int]] = None,
                  retrieved=None) -> Tuple[np.ndarray, np.ndarray]:
    """One decoding step of one sequence (Eq. 2's conditioning on x_<t of the current
    segment, C_{i-1} and R_{i-1}).  q [Hq,D] is the query of the newest token; k_ctx,
    v_ctx [n,Hkv,D] hold the keys/values of all n tokens so far, the newest included.
    By the forward identity of Sec. 3.1 this is row n-1 of the prefill of the same n
    tokens.  retrieved, if given, maps a KV head to the retrieved prefix of the open
    segment.  Returns O [Hq,D] and LSE [Hq]."""
    q = widen(q)
    k_ctx, v_ctx = widen(k_ctx), widen(v_ctx)
    n = k_ctx.shape[0]
    qfull = np.zeros((1, n, q.shape[0], q.shape[1]))
    qfull[0, n - 1] = q
    ret = None if retrieved is None else {(0, h, (n - 1) // seg_len): idx for h, idx in retrieved.items()}
    o, l = attend(qfull, k_ctx[None], v_ctx[None], seg_len=seg_len, tail_len=tail_len,
                  kv_policy=kv_policy, scale=scale, rows=[n - 1], evicted=evicted, retrieved=ret)
    return o[0, 0], l[0, :, 0]


def differentiable_mask(p: int, n: int, seg_len: int, tail_len: int, policy: int) -> np.ndarray:
    """Boolean [n]: the keys of query position p through which gradient flows into K and V.
    The own segment and, for a head with the TAIL bit, the carried tail C_{i-1} (the
    differentiable interface state of Sec. 3.2: with truncation depth K >= 1 the loss of
    segment i reaches the update that produced C_{i-1}).  Past rows reached only through the
    PAST bit are forward-only (Lemma "No-gradient retrieval prefix", Appendix B): they shape
    the softmax but receive no gradient."""
    s = (p // seg_len) * seg_len
    j = np.arange(n)
    diff = (j >= s) & (j <= p)
    if policy & POLICY_TAIL:
        diff |= (j >= max(0, s - tail_len)) & (j < s)
    return diff


def attend_backward(q, k, v, dout, *, seg_len: int, tail_len: int, kv_policy: Sequence[int],
                    scale: Optional[float] = None, evicted: Optional[Sequence[int]] = None,
                    max_block_bytes: int = 1 << 28):
    """Gradients of L = sum(O * dout) for O = attend(q, k, v) (Eq. 12 under the mask of Eq. 13),
    with the stop-gradient placement of Definition "K-truncated consistent objective" and of
    the no-gradient lemma: every visible key contributes to dQ; dK and dV collect only the
    pairs of differentiable_mask().

    With P = softmax(scale * Q K^T + M), dP = dout V^T, delta_i = sum_j P_ij dP_ij and
    dS = P * (dP - delta):   dQ = scale * dS K,   dK = scale * (dS * G)^T Q,   dV = (P * G)^T dout,
    G the 0/1 matrix of differentiable pairs.  q, dout [B,N,Hq,D]; k, v [B,N,Hkv,D]; returns
    dQ [B,N,Hq,D], dK, dV [B,N,Hkv,D] in float64 (the g query heads of a group add up)."""
    q, k, v, dout = widen(q), widen(k), widen(v), widen(dout)
    B, N, Hq, D = q.shape
    Hkv = k.shape[2]
    if k.shape != (B, N, Hkv, D) or v.shape != k.shape or dout.shape != q.shape:
        raise ValueError("shape mismatch")
    if Hq % Hkv or len(kv_policy) != Hkv:
        raise ValueError("bad head configuration")
    g = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    ev = [0] * Hkv if evicted is None else [int(e) for e in evicted]
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    step = max(1, int(max_block_bytes // (8 * max(N, 1))))
    for kvh in range(Hkv):
        pol = int(kv_policy[kvh])
        for r0 in range(0, N, step):
            rr = np.arange(r0, min(N, r0 + step))
            mask = np.stack([visible_mask(int(p), N, seg_len, tail_len, pol, ev[kvh]) for p in rr])
            grad = np.stack([differentiable_mask(int(p), N, seg_len, tail_len, pol) for p in rr])
            for b in range(B):
                kb, vb = k[b, :, kvh, :], v[b, :, kvh, :]
                for h in range(kvh * g, (kvh + 1) * g):
                    z = np.where(mask, (q[b, rr, h, :] @ kb.T) * scale, -np.inf)
                    e = np.exp(z - z.max(axis=1, keepdims=True))
                    pr = e / e.sum(axis=1, keepdims=True)
                    dp = dout[b, rr, h, :] @ vb.T
                    delta = (pr * dp).sum(axis=1, keepdims=True)
                    ds = pr * (dp - delta)
                    dq[b, rr, h, :] = scale * (ds @ kb)
                    dk[b, :, kvh, :] += scale * ((ds * grad).T @ q[b, rr, h, :])
                    dv[b, :, kvh, :] += (pr * grad).T @ dout[b, rr, h, :]
    return dq, dk, dv


def attend_backward_packed(q, k, v, dout, cu_seqlens, **kw):
    """attend_backward for a packed ragged batch (layout as attend_packed): every sequence is
    differentiated on its own; nothing flows across a sequence boundary.  q, dout [total,Hq,D];
    k, v [total,Hkv,D]; returns dQ, dK, dV in the same layouts."""
    dq, dk, dv = np.zeros(q.shape), np.zeros(k.shape), np.zeros(v.shape)
    for b in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        if hi > lo:
            gq, gk, gv = attend_backward(q[None, lo:hi], k[None, lo:hi], v[None, lo:hi], dout[None, lo:hi], **kw)
            dq[lo:hi], dk[lo:hi], dv[lo:hi] = gq[0], gk[0], gv[0]
    return dq, dk, dv


def rope_rotate(x, positions, theta: float = 10000.0) -> np.ndarray:
    """Rotary position embedding of x [..., rows, heads, D] at integer `positions` [rows]
    (standard RoPE, which Appendix E reuses): channel pair (i, i + D/2), i < D/2, is turned by
    the angle position * theta^(-2i/D):  y_i = x_i cos - x_{i+D/2} sin,  y_{i+D/2} = x_i sin +
    x_{i+D/2} cos.  The pairing (first half with second half, as the LLaMA backbones the paper
    uses do) and the base theta are readings: the paper states neither."""
    x = widen(x)
    D = x.shape[-1]
    half = D // 2
    pos = np.asarray(positions, dtype=np.float64).reshape(-1)
    if x.shape[-3] != pos.size or D % 2:
        raise ValueError("positions do not match the rows of x")
    inv_freq = float(theta) ** (-np.arange(half, dtype=np.float64) * 2.0 / D)
    ang = pos[:, None] * inv_freq[None, :]                       # [rows, D/2]
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]  # broadcast over heads
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * cos - b * sin, a * sin + b * cos], axis=-1)


def attend_reindexed(q, k, v, *, seg_len: int, tail_len: int, kv_policy: Sequence[int],
                     theta: float = 10000.0, scale: Optional[float] = None, retrieved=None):
    """Segment-level attention with the RoPE re-indexing of Appendix E, written literally:
    q, k are *unrotated*; for every segment and KV head the prefix the head sees (carried tail,
    whole history, or the retrieved list, in list order) gets key positions 0..P-1 and the
    segment's queries and keys get positions P..P+m-1; values are not rotated.  Returns O
    [B,N,Hq,D] and LSE [B,Hq,N] in float64.  retrieved as in attend()."""
    q, k, v = widen(q), widen(k), widen(v)
    B, N, Hq, D = q.shape
    Hkv = k.shape[2]
    g = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    out = np.zeros((B, N, Hq, D))
    lse = np.zeros((B, Hq, N))
    for b in range(B):
        for kvh in range(Hkv):
            pol = int(kv_policy[kvh])
            for i, s in enumerate(range(0, N, seg_len)):
                m = min(seg_len, N - s)
                if (pol & POLICY_PAST) and retrieved is not None:
                    pref = np.asarray(retrieved.get((b, kvh, i), ()), dtype=np.int64).reshape(-1)
                elif pol & POLICY_PAST:
                    pref = np.arange(0, s)
                elif pol & POLICY_TAIL:
                    pref = np.arange(max(0, s - tail_len), s)
                else:
                    pref = np.arange(0, 0)
                P = pref.size
                kp = rope_rotate(k[b, pref, kvh:kvh + 1, :], np.arange(P), theta)[:, 0]       # prefix keys
                ks = rope_rotate(k[b, s:s + m, kvh:kvh + 1, :], P + np.arange(m), theta)[:, 0]  # segment keys
                kc = np.concatenate([kp, ks])
                vc = np.concatenate([v[b, pref, kvh, :], v[b, s:s + m, kvh, :]])
                for h in range(kvh * g, (kvh + 1) * g):
                    qs = rope_rotate(q[b, s:s + m, h:h + 1, :], P + np.arange(m), theta)[:, 0]
                    z = (qs @ kc.T) * scale
                    allowed = np.concatenate([np.ones((m, P), dtype=bool),
                                              np.tril(np.ones((m, m), dtype=bool))], axis=1)
                    z = np.where(allowed, z, -np.inf)
                    zmax = z.max(axis=1, keepdims=True)
                    e = np.exp(z - zmax)
                    den = e.sum(axis=1, keepdims=True)
                    out[b, s:s + m, h, :] = (e / den) @ vc
                    lse[b, h, s:s + m] = (zmax + np.log(den))[:, 0]
    return out, lse


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 of float64 values, ties to the even significand, returned as float64.

    bfloat16 keeps 8 significant bits (1 sign, 8 exponent, 7 stored fraction bits; the binary32
    exponent range): a value of magnitude in [2^e, 2^(e+1)) lies on a grid of spacing 2^(e-7),
    never finer than the subnormal spacing 2^-133, and what rounds to 2^128 or beyond is
    infinite.  Rounded straight from the float64 value (one rounding, not two)."""
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)                                # |x| in [2^(e-1), 2^e)
    quantum = np.ldexp(1.0, np.maximum(e - 8, -133))  # spacing of the bf16 grid at x
    r = np.rint(x / quantum) * quantum                # rint rounds halves to the even integer
    r = np.where(np.abs(r) >= 2.0 ** 128, np.copysign(np.inf, x), r)
    return np.where(np.isfinite(x), r, x)


def retrieval_summaries(q_prev, *, n_queries: int, pool_window: int, tail_avg: int) -> np.ndarray:
    """Query summaries of Appendix D ("Query construction") for one sequence: from the last
    L = min(n_queries, m) query rows of the previous segment q_prev [m, H, D], (i) the means of
    consecutive windows of pool_window rows (sliding-window mean pooling with stride = window; a
    shorter last window averages what it has) and (ii) the mean of the last min(tail_avg, L)
    rows.  Returns [n_sum, H, D].  Window length, stride and tail length are readings: the paper
    names the two ingredients only."""
    q_prev = widen(q_prev)
    m = q_prev.shape[0]
    L = min(int(n_queries), m)
    last = q_prev[m - L:]
    out = [last[a:a + pool_window].mean(axis=0) for a in range(0, L, pool_window)]
    out.append(last[L - min(int(tail_avg), L):].mean(axis=0))
    return np.stack(out)


def retrieve_indices(q_prev, k_pool, *, R: int, n_queries: int, pool_window: int, tail_avg: int,
                     n_anchors: int, win_before: int, win_after: int, evicted: int = 0,
                     return_scores: bool = False, summaries_bf16: bool = True):
    """Top-k retrieval operator of Appendix D for one sequence and one KV head, as read here.

    q_prev [m, g, D]: previous-segment queries of the g query heads of the group; k_pool [n, D]:
    the head's pool.  Scoring: dot products between every summary and every pool key; a row's
    score is its best over the summaries.  Appendix D fixes no precision for the summaries; by
    default they are rounded to bf16 like every query and key of the bf16 backbones the paper
    runs (Sec. 4), and summaries_bf16=False keeps the float64 means instead.  The two readings
    can only pick different anchors where scores lie within the rounding of each other (each
    score moves by at most 2^-8 sum_d |s_d k_d|); test_oracle_pins checks exactly that.  Anchors: the n_anchors rows with the highest scores (ties: lower row
    first) -- the same rows as "per-summary top-k, de-duplicate, keep the highest-scoring
    anchors" for any k >= n_anchors.  Window expansion: anchors in descending score order each
    add rows a-win_before .. a+win_after (clipped to the pool, ascending, skipping rows already
    in) until R rows are in.  Padding: if fewer than R, the earliest pool rows not yet in.
    Result: the min(R, n - evicted) rows, sorted ascending."""
    q_prev, k_pool = widen(q_prev), widen(k_pool)
    n = k_pool.shape[0]
    summ = retrieval_summaries(q_prev, n_queries=n_queries, pool_window=pool_window, tail_avg=tail_avg)
    if summaries_bf16:
        summ = round_bf16(summ)
    sig = summ.reshape(-1, summ.shape[-1])                  # all summaries of all heads of the group
    scores = (sig @ k_pool.T).max(axis=0)                   # [n]
    scores[:evicted] = -np.inf
    want = min(int(R), n - evicted)
    order = sorted(range(evicted, n), key=lambda r: (-scores[r], r))[:n_anchors]
    chosen = []
    inside = set()
    for a_ in order:
        for r in range(max(evicted, a_ - win_before), min(n, a_ + win_after + 1)):
            if len(chosen) < want and r not in inside:
                inside.add(r)
                chosen.append(r)
    r = evicted
    while len(chosen) < want:
        if r not in inside:
            inside.add(r)
            chosen.append(r)
        r += 1
    res = np.array(sorted(chosen), dtype=np.int64)
    return (res, scores) if return_scores else res


def visible_pairs(n: int, seg_len: int, tail_len: int, policy: int, evicted: int = 0) -> int:
    """Number of (query, key) pairs one head evaluates: popcount of the mask."""
    return int(sum(int(visible_mask(p, n, seg_len, tail_len, policy, evicted).sum())
                   for p in range(n)))


def tail_of(k_seg, v_seg, tail_len: int):
    """Carried state C_i of a finished segment: its last min(T, m) key/value rows."""
    m = k_seg.shape[0]
    t = min(tail_len, m)
    return k_seg[m - t:], v_seg[m - t:]
