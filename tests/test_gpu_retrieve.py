"""GPU checks of the top-k retrieval operator (Appendix D; seg_kv_retrieve) through the C ABI.

The operator ends in integers (row numbers) decided by floating-point scores.  Where the best
scores are far apart (planted keys) the row lists must equal the oracle's exactly; on random
data, where near-ties may fall either way depending on summation order, the lists are checked
for what is unique: shape, order, range, the windows of every clearly winning row, and nothing
that a clearly losing row could explain."""
import numpy as np
import pytest
import torch

import paper_2605_11744_amd as sa
import workloads as W
from gpu_util import Cache, assert_parity, dev_bf16
from oracle import segattn_oracle as orc

pytestmark = pytest.mark.gpu


def _bits(x):
    return W.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def _retrieve(c, params, q_prev_bits, R):
    r = sa.make_retrieval(**params)
    nws = sa.seg_kv_retrieve_workspace_bytes(c.ctx, r)
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    n_past = sum(1 for pol in c.w.kv_policy if pol & 2)
    idx = torch.full((c.B, n_past, R), -1, dtype=torch.int32, device="cuda")
    qp = dev_bf16(q_prev_bits)
    sa.seg_kv_retrieve(c.ctx, r, qp, q_prev_bits.shape[1], R, idx, ws, nws, c.stream)
    torch.cuda.synchronize()
    return idx


def _planted_problem(seed, n, S, D, g, B):
    """k, v random; q_prev rows constant per head (every summary of a head is that vector);
    a few pool rows hold large multiples of head 0's vector: their scores tower over the rest."""
    rng = np.random.default_rng(seed)
    w = W.small(seq_len=n, seg_len=S, tail_len=16, n_q_heads=2 * g, n_kv_heads=2, head_dim=D,
                kv_policy=[2, 1], batch=B)
    q, k, v = W.prefill_inputs(w)
    u = rng.standard_normal((B, 2 * g, D)).astype(np.float32)
    q_prev = np.repeat(_bits(u)[:, None], 24, axis=1)                     # [B, 24, Hq, D]
    planted = {}
    for b in range(B):
        rows = rng.choice(n, size=5, replace=False)
        uf = orc.widen(q_prev[b, 0, 0])                                   # head 0 of KV group 0
        for j, r in enumerate(rows):
            k[b, r, 0] = _bits((30.0 - 3.0 * j) * uf / np.linalg.norm(uf))
        planted[b] = [int(r) for r in rows]
    return w, q, k, v, q_prev, planted


@pytest.mark.parametrize("D,g,params,R,evict", [
    (128, 2, dict(n_queries=24, pool_window=8, tail_avg=4, n_anchors=4, win_before=2, win_after=5), 48, 0),
    (64, 4, dict(n_queries=16, pool_window=4, tail_avg=2, n_anchors=3, win_before=0, win_after=0), 7, 0),
    (128, 1, dict(n_queries=24, pool_window=24, tail_avg=24, n_anchors=5, win_before=8, win_after=8), 30, 100),
    (128, 4, dict(n_queries=64, pool_window=8, tail_avg=8, n_anchors=5, win_before=3, win_after=3), 512, 0),
])
def test_planted_rows_give_exactly_the_oracle_lists(D, g, params, R, evict):
    n, S, B = 768, 128, 2
    w, q, k, v, q_prev, planted = _planted_problem(D + g, n, S, D, g, B)
    c = Cache(w, past_capacity=1024, fp32_check=True)
    try:
        for s in range(0, n, S):
            c.fwd(q[:, s:s + S], k[:, s:s + S], v[:, s:s + S])
        if evict:
            sa.seg_kv_past_evict(c.ctx, 0, evict, c.stream)
        idx = _retrieve(c, params, q_prev, R).cpu().numpy()
    finally:
        c.close()
    for b in range(B):
        want = orc.retrieve_indices(q_prev[b, :, :g], k[b, :, 0], R=R, evicted=evict, **params)
        assert list(idx[b, 0]) == list(want), (b, planted[b])


def test_random_scores_lists_are_valid():
    n, S, B, D, g, R = 1024, 256, 2, 128, 4, 96
    params = dict(n_queries=32, pool_window=8, tail_avg=4, n_anchors=6, win_before=4, win_after=4)
    w = W.small(seq_len=n + S, seg_len=S, tail_len=32, n_q_heads=2 * g, n_kv_heads=2, head_dim=D,
                kv_policy=[1, 2], batch=B)
    q, k, v = W.prefill_inputs(w)
    c = Cache(w, past_capacity=2048, fp32_check=True)
    try:
        for s in range(0, n, S):
            c.fwd(q[:, s:s + S], k[:, s:s + S], v[:, s:s + S])
        q_prev = q[:, n - S:n]
        idx = _retrieve(c, params, q_prev, R).cpu().numpy()
    finally:
        c.close()
    span = params["win_before"] + params["win_after"] + 1
    assert params["n_anchors"] * span <= R                      # no truncation in this configuration
    for b in range(B):
        got = idx[b, 0]
        assert len(set(got.tolist())) == R and (np.diff(got) > 0).all() and got[0] >= 0 and got[-1] < n
        _, sc = orc.retrieve_indices(q_prev[b, :, g:2 * g], k[b, :n, 1], R=R, return_scores=True, **params)
        nth = np.sort(sc)[-params["n_anchors"]]
        eps = 0.5
        def windows(rows):
            out = set()
            for a_ in rows:
                out |= set(range(max(0, a_ - params["win_before"]), min(n, a_ + params["win_after"] + 1)))
            return out
        sure, maybe = np.nonzero(sc > nth + eps)[0], np.nonzero(sc >= nth - eps)[0]
        assert windows(sure) <= set(got.tolist())
        rest = set(got.tolist()) - windows(maybe)
        assert all(r < R for r in rest)                          # padding: among the earliest rows


def test_retrieve_then_select_then_attend_matches_oracle():
    n, S, B, D, g, R = 512, 128, 2, 128, 2, 40
    params = dict(n_queries=24, pool_window=8, tail_avg=4, n_anchors=4, win_before=2, win_after=5)
    w, q, k, v, q_prev, _ = _planted_problem(11, n + S, S, D, g, B)
    c = Cache(w, past_capacity=1024, fp32_check=True, retrieved_capacity=R)
    try:
        for s in range(0, n, S):
            c.fwd(q[:, s:s + S], k[:, s:s + S], v[:, s:s + S])
        idx = _retrieve(c, params, q_prev, R)
        sa.seg_kv_past_select(c.ctx, idx, R, c.stream)
        o, l = c.fwd(q[:, n:], k[:, n:], v[:, n:])
    finally:
        c.close()
    retrieved = {(b, 0, n // S): orc.retrieve_indices(q_prev[b, :, :g], k[b, :n, 0], R=R, **params) for b in range(B)}
    o_ref, l_ref = orc.attend(q, k, v, seg_len=S, tail_len=16, kv_policy=w.kv_policy, retrieved=retrieved,
                              rows=list(range(n, n + S)))
    assert_parity(o, l, o_ref, l_ref, fp32_check=True, what="retrieve + select + fwd")


def test_retrieve_validation():
    w = W.small(seq_len=256, seg_len=128, tail_len=16, n_q_heads=8, n_kv_heads=2, head_dim=64, kv_policy=[2, 1])
    q, k, v = W.prefill_inputs(w)
    c = Cache(w, past_capacity=512, fp32_check=True)
    good = dict(n_queries=24, pool_window=8, tail_avg=4, n_anchors=4, win_before=2, win_after=2)
    try:
        assert sa.seg_kv_retrieve_workspace_bytes(c.ctx, sa.make_retrieval(**{**good, "n_anchors": 33})) == 0
        assert sa.seg_kv_retrieve_workspace_bytes(c.ctx, sa.make_retrieval(**{**good, "pool_window": 1})) == 0  # 25 summaries x 4 heads
        r = sa.make_retrieval(**good)
        nws = sa.seg_kv_retrieve_workspace_bytes(c.ctx, r)
        ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
        idx = torch.empty((1, 1, 8), dtype=torch.int32, device="cuda")
        with pytest.raises(sa.SegattnError) as e:                     # empty pool
            sa.seg_kv_retrieve(c.ctx, r, dev_bf16(q[:, :128]), 128, 8, idx, ws, nws, c.stream)
        assert e.value.status == sa.SEGATTN_ECAPACITY
        c.fwd(q[:, :128], k[:, :128], v[:, :128])
        with pytest.raises(sa.SegattnError) as e:                     # workspace too small
            sa.seg_kv_retrieve(c.ctx, r, dev_bf16(q[:, :128]), 128, 8, idx, ws, nws - 256, c.stream)
        assert e.value.status == sa.SEGATTN_EINVAL
    finally:
        c.close()
