"""GPU parity of the retrieval mode (Sec. 3.4 "Long-Range Channel"; Eq. 13, second case;
Appendix D "Output"): a long-range head attends to [R gathered pool rows ; own segment].
Every case runs the library segment by segment through the C ABI -- seg_kv_past_select,
seg_attn_fwd, seg_kv_commit, seg_attn_decode -- and compares with the fp64 oracle given the
same index lists."""
import numpy as np
import pytest
import torch

import paper_2605_11744_amd as sa
import workloads as W
from gpu_util import Cache, assert_parity
from oracle import segattn_oracle as orc

pytestmark = pytest.mark.gpu


def _lists(rng, B, past_heads, pool_rows, R):
    """[B, n_past, R] distinct pool rows in random order, plus the oracle's dictionary entries."""
    idx = np.stack([np.stack([rng.permutation(pool_rows)[:R] for _ in past_heads]) for _ in range(B)])
    return idx.astype(np.int32)


def _run_prefill(w, n, R, chunks, fp32_check, seed):
    q, k, v = W.prefill_inputs(w, seq_len=n)
    B, S = w.batch, w.seg_len
    past_heads = [h for h, pol in enumerate(w.kv_policy) if pol & 2]
    rng = np.random.default_rng(seed)
    c = Cache(w, past_capacity=((n + S - 1) // S) * S, fp32_check=fp32_check, retrieved_capacity=max(R, 1))
    retrieved = {}
    o_parts, l_parts = [], []
    try:
        for i, s in enumerate(range(0, n, S)):
            m = min(S, n - s)
            r = min(R, s)
            if r > 0:
                idx = _lists(rng, B, past_heads, s, r)
                c.select(idx)
                for b in range(B):
                    for j, h in enumerate(past_heads):
                        retrieved[(b, h, i)] = idx[b, j]
            cuts = [0] + [x for x in chunks if x < m] + [m]
            for a, e in zip(cuts[:-1], cuts[1:]):
                o, l = c.fwd(q[:, s + a:s + e], k[:, s + a:s + e], v[:, s + a:s + e])
                o_parts.append(o)
                l_parts.append(l)
        resident = sa.segattn_resident_bytes(c.ctx)
    finally:
        c.close()
    o_gpu, l_gpu = np.concatenate(o_parts, axis=1), np.concatenate(l_parts, axis=2)
    o_ref, l_ref = orc.attend(q, k, v, seg_len=S, tail_len=w.tail_len, kv_policy=w.kv_policy, retrieved=retrieved)
    return o_gpu, l_gpu, o_ref, l_ref, resident


@pytest.mark.parametrize("fp32_check", [True, False])
@pytest.mark.parametrize("D,g,R,n,chunks", [
    (128, 4, 48, 700, ()),            # whole segments, ragged last one
    (64, 2, 100, 640, (37,)),         # segment fed in two calls: prefix + committed rows + new rows
    (128, 1, 5, 521, (64, 65)),       # tiny prefix, three calls per segment
])
def test_retrieval_mode_prefill_matches_oracle(fp32_check, D, g, R, n, chunks):
    w = W.small(seq_len=n, seg_len=128, tail_len=32, n_q_heads=4 * g, n_kv_heads=4, head_dim=D,
                kv_policy=[1, 2, 0, 2], batch=2)
    o_gpu, l_gpu, o_ref, l_ref, resident = _run_prefill(w, n, R, chunks, fp32_check, seed=D + n)
    assert_parity(o_gpu, l_gpu, o_ref, l_ref, fp32_check=fp32_check, what=f"retrieval D={D} R={R}")
    assert resident > 0


def test_retrieval_with_full_lists_equals_full_history_library_result():
    """Selecting every pool row must reproduce what the library computes for a PAST head that
    reads its whole pool (two different code paths of the library, one oracle)."""
    n, S = 512, 128
    w = W.small(seq_len=n, seg_len=S, tail_len=32, n_q_heads=4, n_kv_heads=2, head_dim=128,
                kv_policy=[2, 1], batch=1)
    q, k, v = W.prefill_inputs(w)
    outs = {}
    for mode in ("pool", "lists"):
        c = Cache(w, past_capacity=n, fp32_check=True, retrieved_capacity=n if mode == "lists" else 0)
        try:
            parts = []
            for s in range(0, n, S):
                if mode == "lists" and s:
                    c.select(np.arange(s, dtype=np.int32)[None, None, :])
                parts.append(c.fwd(q[:, s:s + S], k[:, s:s + S], v[:, s:s + S]))
            outs[mode] = (np.concatenate([p[0] for p in parts], 1), np.concatenate([p[1] for p in parts], 2))
        finally:
            c.close()
    np.testing.assert_allclose(outs["lists"][0], outs["pool"][0], atol=2e-5)
    np.testing.assert_allclose(outs["lists"][1], outs["pool"][1], atol=2e-5)


@pytest.mark.parametrize("fp32_check", [True, False])
def test_retrieval_mode_decode_crosses_a_segment_boundary(fp32_check):
    S, T, R, n0, steps = 64, 16, 24, 150, 60       # decode rows 150..209: boundary at 192
    w = W.small(seq_len=n0 + steps, seg_len=S, tail_len=T, n_q_heads=8, n_kv_heads=2, head_dim=128,
                kv_policy=[2, 1], batch=2)
    q, k, v = W.prefill_inputs(w)
    rng = np.random.default_rng(7)
    c = Cache(w, past_capacity=256, fp32_check=fp32_check, retrieved_capacity=R)
    retrieved = {}
    def select_for(i):
        idx = _lists(rng, 2, [0], i * S, min(R, i * S))
        c.select(idx)
        for b in range(2):
            retrieved[(b, 0, i)] = idx[b, 0]
    try:
        for i, s in enumerate(range(0, n0, S)):
            if i:
                select_for(i)
            e = min(n0, s + S)
            c.fwd(q[:, s:e], k[:, s:e], v[:, s:e])
        o_rows, l_rows = [], []
        for t in range(n0, n0 + steps):
            if t % S == 0:
                select_for(t // S)
            o, l = c.decode(q[:, t], k[:, t], v[:, t])
            o_rows.append(o)
            l_rows.append(l)
    finally:
        c.close()
    o_gpu, l_gpu = np.stack(o_rows, axis=1), np.stack(l_rows, axis=2)
    o_ref, l_ref = orc.attend(q, k, v, seg_len=S, tail_len=T, kv_policy=w.kv_policy, retrieved=retrieved,
                              rows=list(range(n0, n0 + steps)))
    assert_parity(o_gpu, l_gpu, o_ref, l_ref, fp32_check=fp32_check, what="retrieval decode")


def test_select_state_errors_and_out_of_range_entries_are_safe():
    S = 64
    w = W.small(seq_len=3 * S, seg_len=S, tail_len=8, n_q_heads=2, n_kv_heads=2, head_dim=64,
                kv_policy=[2, 1], batch=1)
    q, k, v = W.prefill_inputs(w)
    c = Cache(w, past_capacity=4 * S, fp32_check=True, retrieved_capacity=16)
    try:
        with pytest.raises(sa.SegattnError) as e:           # empty pool cannot serve 4 rows
            c.select(np.zeros((1, 1, 4), dtype=np.int32))
        assert e.value.status == sa.SEGATTN_ECAPACITY
        c.fwd(q[:, :S], k[:, :S], v[:, :S])
        c.fwd(q[:, S:S + 10], k[:, S:S + 10], v[:, S:S + 10])
        with pytest.raises(sa.SegattnError) as e:           # a segment is open
            c.select(np.zeros((1, 1, 4), dtype=np.int32))
        assert e.value.status == sa.SEGATTN_ESTATE
        c.fwd(q[:, S + 10:2 * S], k[:, S + 10:2 * S], v[:, S + 10:2 * S])
        # entries outside the pool are clamped to its first / last row: same result as naming those rows
        c.select(np.array([[[-5, 3, 1 << 30]]], dtype=np.int32))
        o, l = c.fwd(q[:, 2 * S:], k[:, 2 * S:], v[:, 2 * S:])
    finally:
        c.close()
    o_ref, l_ref = orc.attend(q, k, v, seg_len=S, tail_len=8, kv_policy=w.kv_policy,
                              retrieved={(0, 0, 2): [0, 3, 2 * S - 1]}, rows=list(range(2 * S, 3 * S)))
    assert_parity(o, l, o_ref, l_ref, fp32_check=True, what="clamped lists")
