"""GPU parity for the stateful path: seg_attn_fwd + seg_kv_commit segment by segment,
tail hand-off, past pool append / evict, and decode steps, against the fp64 oracle."""
import numpy as np
import pytest

import workloads as W
from oracle import segattn_oracle as orc

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _oracle(w, q, k, v, **kw):
    return orc.attend(q, k, v, seg_len=w.seg_len, tail_len=w.tail_len, kv_policy=w.kv_policy, **kw)


STREAM_CASES = [
    # (workload kwargs, chunk sizes cycled through while streaming)
    (dict(seq_len=300, seg_len=64, tail_len=16, n_q_heads=8, n_kv_heads=4, head_dim=128), [64]),
    (dict(seq_len=300, seg_len=64, tail_len=64, n_q_heads=4, n_kv_heads=4, head_dim=64), [64]),
    (dict(seq_len=520, seg_len=128, tail_len=40, n_q_heads=16, n_kv_heads=4, head_dim=128, batch=2), [50, 78, 128, 1, 127]),
    (dict(seq_len=257, seg_len=256, tail_len=0, n_q_heads=8, n_kv_heads=4, head_dim=64), [200, 56, 1]),
    # prefixes of thousands of rows: the library cuts a PAST head's prefix into 2 to 4 pieces per
    # query block (separate workgroups, merged afterwards), also with a partly filled open segment
    (dict(seq_len=5500, seg_len=1024, tail_len=128, n_q_heads=8, n_kv_heads=2, head_dim=128, kv_policy=[3, 1],
          batch=2), [1024, 600, 424]),
    (dict(seq_len=3400, seg_len=512, tail_len=64, n_q_heads=4, n_kv_heads=2, head_dim=128, kv_policy=[2, 1]),
     [512, 100, 412]),
]


@pytest.mark.parametrize("waves", ["auto", "4", "8", "queue"])
@pytest.mark.parametrize("fp32_check", [True, False])
@pytest.mark.parametrize("case", range(len(STREAM_CASES)))
def test_streaming_prefill_equals_oracle(case, fp32_check, waves, monkeypatch):
    import gpu_util as G
    kw, chunks = STREAM_CASES[case]
    if waves == "queue":   # the library's own workgroup shape, work items taken from queues
        if fp32_check:
            pytest.skip("the item queues only exist in the MFMA kernel")
        monkeypatch.setitem(G.TUNING, "item_queues", G.QUEUES_ON_SMALL_GRID)
    elif waves != "auto":
        if fp32_check or kw["head_dim"] != 128:
            pytest.skip("the wave count only exists in the head_dim-128 MFMA kernel")
        monkeypatch.setitem(G.TUNING, "prefill_waves", int(waves))
    w = W.small(f"stream{case}", index=200 + case, **kw)
    q, k, v = W.prefill_inputs(w)
    o_ref, l_ref = _oracle(w, q, k, v)
    c = G.Cache(w, past_capacity=((w.seq_len + w.seg_len) // w.seg_len) * w.seg_len, fp32_check=fp32_check)
    try:
        o = np.zeros_like(o_ref)
        l = np.zeros_like(l_ref)
        pos, i = 0, 0
        while pos < w.seq_len:
            room = w.seg_len - pos % w.seg_len
            m = min(chunks[i % len(chunks)], room, w.seq_len - pos)
            i += 1
            oc, lc = c.fwd(q[:, pos:pos + m], k[:, pos:pos + m], v[:, pos:pos + m])
            o[:, pos:pos + m] = oc
            l[:, :, pos:pos + m] = lc
            pos += m
        G.assert_parity(o, l, o_ref, l_ref, fp32_check=fp32_check, what=f"stream{case}")
        # counters: closed segments, tail, open segment, resident rows (Sec. 3.5 memory bound)
        import paper_2605_11744_amd as sa
        past, tail, fill = sa.seg_kv_lengths(c.ctx, c.B, w.n_kv_heads)
        closed = (w.seq_len // w.seg_len) * w.seg_len
        exp_tail = w.tail_len if closed else 0
        assert fill == [w.seq_len - closed] * c.B and tail == [exp_tail] * c.B
        rows = 0
        for h, pol in enumerate(w.kv_policy):
            assert all(past[b][h] == (closed if pol & 2 else 0) for b in range(c.B))
            rows += (closed if pol & 2 else (exp_tail if pol & 1 else 0)) + (w.seq_len - closed)
        assert sa.segattn_resident_bytes(c.ctx) == c.B * rows * 2 * w.head_dim * 2
    finally:
        c.close()


@pytest.mark.parametrize("fp32_check", [True, False])
def test_decode_after_prefill_crosses_segment_boundaries(fp32_check):
    """Prefill n0 tokens, then decode token by token across two segment closures: every step
    must equal the oracle's row for that position (forward identity, Sec. 3.1)."""
    import gpu_util as G
    w = W.small("dec_after_prefill", index=210, seq_len=200, seg_len=48, tail_len=20, n_q_heads=8,
                n_kv_heads=4, head_dim=128, batch=2)
    q, k, v = W.prefill_inputs(w)
    o_ref, l_ref = _oracle(w, q, k, v)
    n0 = 70
    c = G.Cache(w, past_capacity=240, fp32_check=fp32_check)
    try:
        pos = 0
        while pos < n0:
            m = min(w.seg_len - pos % w.seg_len, n0 - pos)
            c.fwd(q[:, pos:pos + m], k[:, pos:pos + m], v[:, pos:pos + m])
            pos += m
        o = np.zeros_like(o_ref[:, n0:])
        l = np.zeros_like(l_ref[:, :, n0:])
        for p in range(n0, w.seq_len):
            od, ld = c.decode(q[:, p], k[:, p], v[:, p])
            o[:, p - n0] = od
            l[:, :, p - n0] = ld
        G.assert_parity(o, l, o_ref[:, n0:], l_ref[:, :, n0:], fp32_check=fp32_check, what="decode steps")
    finally:
        c.close()


def _decode_from_restored_cache(w, k_done, c_fill, fp32_check=False):
    """Rows written into the arena through segattn_cache_span, lengths declared with
    seg_kv_set_lengths, one decode step checked against the decode oracle per sequence."""
    import gpu_util as G
    import paper_2605_11744_amd as sa
    S, T, B, Hkv, D = w.seg_len, w.tail_len, w.batch, w.n_kv_heads, w.head_dim
    q, ks, vs, _, _ = W.decode_inputs(w, k_done, c_fill)      # whole histories: the oracle sees every row
    c = G.Cache(w, past_capacity=w.max_context, fp32_check=fp32_check)
    try:
        k_new, v_new = G.fill_cache_for_decode(c, w, ks, vs, k_done, c_fill)
        o, l = c.decode(q, k_new, v_new)
        for b in range(B):
            n_b = int(k_done[b]) * S + int(c_fill[b])
            kf, vf = G.full_history(ks[b], vs[b], n_b, Hkv, D)
            o_ref, l_ref = orc.decode_attend(q[b], kf, vf, seg_len=S, tail_len=T, kv_policy=w.kv_policy)
            G.assert_parity(o[b], l[b], o_ref, l_ref, fp32_check=fp32_check, what=f"{w.name} decode b={b}")
        return sa.seg_kv_lengths(c.ctx, B, Hkv)
    finally:
        c.close()


def test_decode_ragged_batch_from_restored_cache():
    """Sequences of different lengths, one of them filling its segment with this token."""
    S, T = 64, 24
    w = W.Workload("dec_ragged", 220, 3, 0, 16, 4, 128, S, T, (1, 3, 0, 2), decode=True, max_context=64 * 9)
    past, tail, fill = _decode_from_restored_cache(w, np.array([1, 8, 3]), np.array([64, 1, 37]))
    # sequence 0 filled its segment with this token: it must have been closed
    assert fill == [0, 1, 37] and past[0][1] == 128 and past[0][3] == 128


@pytest.mark.parametrize("n_q_heads,head_dim,fp32_check", [(16, 128, False), (8, 128, False), (4, 64, False),
                                                           (32, 64, False), (32, 128, False), (12, 128, False),
                                                           (16, 128, True), (32, 128, True), (20, 128, False),
                                                           (28, 64, False), (48, 128, False), (28, 128, True),
                                                           (64, 128, False), (64, 64, False), (96, 128, False)])
def test_decode_slices_cut_windows_anywhere(n_q_heads, head_dim, fp32_check):
    """Windows of 1 to ~2800 rows (about 17K rows in all): the split kernel's equal slices of 512
    rows begin and end inside windows, cover several short windows at once, and a long window
    gets partials from several workgroups; GQA group sizes 1, 2, 3, 4, 5, 7, 8, 12, 16 and 24 (the
    matrix-core split kernel takes up to 16 heads per pass, the fp32 one 1, 2, 4 or 8; a group that
    does not fill its last pass computes surplus heads and drops them)."""
    S, T = 256, 100
    w = W.Workload("dec_slices", 221, 5, 0, n_q_heads, 4, head_dim, S, T, (1, 3, 0, 2), decode=True,
                   max_context=S * 12)
    _decode_from_restored_cache(w, np.array([1, 11, 3, 7, 5]), np.array([256, 1, 37, 200, 129]), fp32_check)


def test_evict_hides_oldest_pool_rows():
    import gpu_util as G
    import paper_2605_11744_amd as sa
    w = W.small("evict", index=230, seq_len=256, seg_len=64, tail_len=16, n_q_heads=4, n_kv_heads=2,
                head_dim=64, kv_policy=[3, 2])
    q, k, v = W.prefill_inputs(w)
    c = G.Cache(w, past_capacity=256)
    try:
        for s in range(0, 192, 64):
            c.fwd(q[:, s:s + 64], k[:, s:s + 64], v[:, s:s + 64])
        sa.seg_kv_past_evict(c.ctx, 0, 100, c.stream)
        sa.seg_kv_past_evict(c.ctx, 1, 50, c.stream)
        sa.seg_kv_past_evict(c.ctx, 0, 1000, c.stream)   # clamps at the tail window: 192 - 16
        o, l = c.fwd(q[:, 192:], k[:, 192:], v[:, 192:])
        o_ref, l_ref = _oracle(w, q, k, v, rows=np.arange(192, 256), evicted=[192, 50])
        G.assert_parity(o, l, o_ref, l_ref, fp32_check=False, what="evict")
        past, _, _ = sa.seg_kv_lengths(c.ctx, 1, 2)
        assert past[0] == [256 - 176, 256 - 50]      # the last fwd committed a fourth segment
    finally:
        c.close()


def test_evicting_more_rows_than_any_count_hides_the_whole_pool():
    """n_oldest up to INT64_MAX after an earlier eviction (the first visible row is no longer 0, so
    first + n must not wrap): everything goes, except the tail window of a TAIL|PAST head; device
    counters and the host's bookkeeping agree (the next segment matches the oracle)."""
    import gpu_util as G
    import paper_2605_11744_amd as sa
    w = W.small("evict_all", index=231, seq_len=256, seg_len=64, tail_len=16, n_q_heads=4, n_kv_heads=2,
                head_dim=64, kv_policy=[3, 2])
    q, k, v = W.prefill_inputs(w)
    c = G.Cache(w, past_capacity=256)
    try:
        for s in range(0, 192, 64):
            c.fwd(q[:, s:s + 64], k[:, s:s + 64], v[:, s:s + 64])
        sa.seg_kv_past_evict(c.ctx, 0, 7, c.stream)
        sa.seg_kv_past_evict(c.ctx, 1, 9, c.stream)
        for h in (0, 1):
            sa.seg_kv_past_evict(c.ctx, h, 2 ** 63 - 1, c.stream)
        past, _, _ = sa.seg_kv_lengths(c.ctx, 1, 2)
        assert past[0] == [16, 0]
        o, l = c.fwd(q[:, 192:], k[:, 192:], v[:, 192:])
        o_ref, l_ref = _oracle(w, q, k, v, rows=np.arange(192, 256), evicted=[192, 192])
        G.assert_parity(o, l, o_ref, l_ref, fp32_check=False, what="evict everything")
    finally:
        c.close()


def test_keep_recent_holds_a_sliding_budget_of_pool_rows():
    """seg_kv_past_keep_recent after every commit: the PAST head sees at most `budget` rows before
    its segment; the oracle models that as evicted = s - budget per segment."""
    import gpu_util as G
    import paper_2605_11744_amd as sa
    S, budget = 64, 100
    w = W.small("budget", index=231, seq_len=320, seg_len=S, tail_len=16, n_q_heads=4, n_kv_heads=2,
                head_dim=128, kv_policy=[2, 3], batch=2)
    q, k, v = W.prefill_inputs(w)
    c = G.Cache(w, past_capacity=320)
    try:
        for s in range(0, 320, S):
            o, l = c.fwd(q[:, s:s + S], k[:, s:s + S], v[:, s:s + S])
            ev = max(0, s - budget)
            o_ref, l_ref = _oracle(w, q, k, v, rows=np.arange(s, s + S), evicted=[ev, ev])
            G.assert_parity(o, l, o_ref, l_ref, fp32_check=False, what=f"budget, segment at {s}")
            sa.seg_kv_past_keep_recent(c.ctx, 0, budget, c.stream)
            sa.seg_kv_past_keep_recent(c.ctx, 1, budget, c.stream)
        past, _, _ = sa.seg_kv_lengths(c.ctx, 2, 2)
        assert past == [[budget, budget], [budget, budget]]
        sa.seg_kv_past_keep_recent(c.ctx, 1, 3, c.stream)      # the tail window (16 rows) stays
        sa.seg_kv_past_keep_recent(c.ctx, 0, 3, c.stream)
        past, _, _ = sa.seg_kv_lengths(c.ctx, 2, 2)
        assert past == [[3, 16], [3, 16]]
    finally:
        c.close()


def test_past_append_explicit_rows_act_as_prefix():
    """Rows handed to seg_kv_past_append become the long-range prefix of the next segment
    (Eq. 13, second case, with gathered rows in place of the whole history)."""
    import gpu_util as G
    import paper_2605_11744_amd as sa
    R = 40
    w = W.small("append", index=240, seq_len=128, seg_len=64, tail_len=R, n_q_heads=4, n_kv_heads=1,
                head_dim=128, kv_policy=[2])
    q, k, v = W.prefill_inputs(w)
    c = G.Cache(w, past_capacity=192)
    try:
        kp = G.dev_bf16(k[:, 64 - R:64, 0])
        vp = G.dev_bf16(v[:, 64 - R:64, 0])
        sa.seg_kv_past_append(c.ctx, 0, kp, vp, R, c.stream)
        o, l = c.fwd(q[:, 64:], k[:, 64:], v[:, 64:])
        # the same rows seen as a carried tail of length R by the oracle
        o_ref, l_ref = orc.attend(q, k, v, seg_len=64, tail_len=R, kv_policy=[1], rows=np.arange(64, 128))
        G.assert_parity(o, l, o_ref, l_ref, fp32_check=False, what="past_append")
    finally:
        c.close()


@pytest.mark.parametrize("n,retrieved", [(300, 0), (256, 0), (50, 0), (641, 0), (300, 48), (384, 48)])
def test_whole_prompt_commit_leaves_the_state_of_per_segment_commits(n, retrieved):
    """seg_kv_commit_seq against a chain of seg_kv_commit calls: same counters, and the same decode
    step and next prefill chunk afterwards (bit for bit: both read the same rows), also on top of
    an earlier segment and in retrieval mode; and the decode row against the oracle."""
    import gpu_util as G
    import paper_2605_11744_amd as sa
    S, T, first = 128, 40, 128
    policy = [2, 1, 0, 2] if retrieved else [3, 1, 0, 2]
    w = W.small("bulk", index=260, seq_len=first + n + 25, seg_len=S, tail_len=T, n_q_heads=8, n_kv_heads=4,
                head_dim=128, kv_policy=policy, batch=2)
    q, k, v = W.prefill_inputs(w)
    caches = [G.Cache(w, past_capacity=1024, retrieved_capacity=retrieved) for _ in range(2)]
    try:
        outs = []
        for which, c in enumerate(caches):
            kd, vd = G.dev_bf16(k), G.dev_bf16(v)
            sa.seg_kv_commit(c.ctx, kd[:, :first].contiguous(), vd[:, :first].contiguous(), first, c.stream)
            if which == 0:
                sa.seg_kv_commit_seq(c.ctx, kd[:, first:first + n].contiguous(), vd[:, first:first + n].contiguous(), n, c.stream)
            else:
                pos = first
                while pos < first + n:
                    m = min(S - (pos - first) % S, first + n - pos)
                    sa.seg_kv_commit(c.ctx, kd[:, pos:pos + m].contiguous(), vd[:, pos:pos + m].contiguous(), m, c.stream)
                    pos += m
            lengths = sa.seg_kv_lengths(c.ctx, 2, 4)
            if retrieved and n % S == 0:   # a selection needs a segment boundary; a close drops the last one
                idx = np.tile(np.arange(retrieved, dtype=np.int32)[None, None], (2, 2, 1)) * 2   # rows 0, 2, 4, ...
                c.select(idx)
            p = first + n
            od, ld = c.decode(q[:, p], k[:, p], v[:, p])
            oc, lc = c.fwd(q[:, p + 1:p + 25], k[:, p + 1:p + 25], v[:, p + 1:p + 25])
            outs.append((lengths, od, ld, oc, lc))
        assert outs[0][0] == outs[1][0]
        for a, b in zip(outs[0][1:], outs[1][1:]):
            np.testing.assert_array_equal(a, b)
        if not retrieved:
            o_ref, l_ref = orc.attend(q, k, v, seg_len=S, tail_len=T, kv_policy=policy, rows=[first + n])
            G.assert_parity(outs[0][1], outs[0][2], o_ref[:, 0], l_ref[:, :, 0], fp32_check=False, what="decode after bulk commit")
            o_ref, l_ref = orc.attend(q, k, v, seg_len=S, tail_len=T, kv_policy=policy, rows=list(range(first + n + 1, first + n + 25)))
            G.assert_parity(outs[0][3], outs[0][4], o_ref, l_ref, fp32_check=False, what="chunk after bulk commit")
    finally:
        for c in caches:
            c.close()


def test_whole_prompt_commit_rejects_an_open_segment_and_an_overfull_pool():
    import gpu_util as G
    import paper_2605_11744_amd as sa
    w = W.small("bulk_err", index=261, seq_len=400, seg_len=128, tail_len=32, n_q_heads=4, n_kv_heads=2,
                head_dim=64, kv_policy=[3, 1])
    _, k, v = W.prefill_inputs(w)
    c = G.Cache(w, past_capacity=256)
    try:
        kd, vd = G.dev_bf16(k), G.dev_bf16(v)
        with pytest.raises(sa.SegattnError):   # 400 rows do not fit a pool of 256
            sa.seg_kv_commit_seq(c.ctx, kd, vd, 400, c.stream)
        sa.seg_kv_commit(c.ctx, kd[:, :10].contiguous(), vd[:, :10].contiguous(), 10, c.stream)
        with pytest.raises(sa.SegattnError):   # a segment is open
            sa.seg_kv_commit_seq(c.ctx, kd[:, 10:100].contiguous(), vd[:, 10:100].contiguous(), 90, c.stream)
        assert sa.seg_kv_lengths(c.ctx, 1, 2) == ([[0, 0]], [0], [10])   # refused calls changed nothing
    finally:
        c.close()


def test_decode_many_short_windows():
    """600 windows of 1 to 100 rows: every thread of a split workgroup sums a run of several windows
    to find where its slice starts, and one slice covers dozens of whole windows."""
    S, T, B = 32, 8, 150
    w = W.Workload("dec_many", 222, B, 0, 8, 4, 64, S, T, (1, 3, 0, 2), decode=True, max_context=S * 4)
    rng = np.random.default_rng(222)
    _decode_from_restored_cache(w, rng.integers(1, 3, size=B), rng.integers(1, S + 1, size=B))
