"""GPU parity at the benchmark's full sizes and launch configuration: the library runs the
whole workload exactly as bench.py does (bf16 output, one seg_attn_fwd_seq launch; the
B=64 decode step), and the fp64 oracle recomputes a sample of the outputs one by one.
Properties that hold at any size (finite, inside the convex hull of V) cover the rest."""
import numpy as np
import pytest

import workloads as W
from oracle import segattn_oracle as orc

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _sample_rows(w, n_random, seed):
    S, T, N = w.seg_len, w.tail_len, w.seq_len
    fixed = {0, 1, 31, 32, 63, 64, S - 1, S, S + 1, S + T - 1, S + T, 2 * S - 1, 2 * S, N // 2 - 1, N // 2,
             N - S, N - S + 1, N - 65, N - 64, N - 1}
    rng = np.random.default_rng(seed)
    rows = sorted({r for r in fixed if 0 <= r < N} | set(int(x) for x in rng.integers(0, N, n_random)))
    return np.array(rows, dtype=np.int64)


def _check_rows(w, q, k, v, o_gpu, l_gpu, rows, bf16_out):
    """o_gpu [B,R,Hq,D], l_gpu [B,Hq,R] are the GPU results at `rows`."""
    o_ref, l_ref = orc.attend(q, k, v, seg_len=w.seg_len, tail_len=w.tail_len, kv_policy=w.kv_policy, rows=rows)
    eo, el = np.abs(o_gpu - o_ref), np.abs(l_gpu - l_ref)
    # a bf16 result carries its own rounding (half an ulp: 2^-9 relative) on top of the 1e-2 bar
    slack = np.abs(o_ref) * 2.0 ** -8 if bf16_out else 0.0
    assert np.all(eo <= 1e-2 + slack), f"O max-abs {eo.max():.3e}"
    assert eo.mean() <= 1e-3, f"O mean-abs {eo.mean():.3e}"
    assert el.max() <= 1e-2 and el.mean() <= 1e-3, f"LSE max {el.max():.3e} mean {el.mean():.3e}"
    return eo.max(), eo.mean(), el.max()


def _run_full(w, bf16_out):
    import gpu_util as G
    import paper_2605_11744_amd as sa
    q, k, v = W.prefill_inputs(w)
    cfg = G.config_of(w, out_fp32=not bf16_out)
    qd, kd, vd = G.dev_bf16(q), G.dev_bf16(k), G.dev_bf16(v)
    odt = torch.bfloat16 if bf16_out else torch.float32
    out = torch.full((w.batch, w.seq_len, w.n_q_heads, w.head_dim), float("nan"), dtype=odt, device="cuda")
    lse = torch.full((w.batch, w.n_q_heads, w.seq_len), float("nan"), dtype=torch.float32, device="cuda")
    sa.seg_attn_fwd_seq(cfg, qd, kd, vd, w.seq_len, out, lse, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    # properties at any size: everything written, finite, O inside the convex hull of V per KV head
    assert bool(torch.isfinite(out).all()) and bool(torch.isfinite(lse).all())
    vmax = vd.float().amax(dim=1).repeat_interleave(w.group, dim=1)      # [B, Hq, D]
    vmin = vd.float().amin(dim=1).repeat_interleave(w.group, dim=1)
    of = out.float()
    tol = 0.04 if bf16_out else 1e-3
    assert bool((of <= vmax[:, None] + tol).all()) and bool((of >= vmin[:, None] - tol).all())
    return q, k, v, out, lse


@pytest.mark.parametrize("name,n_random,bf16_out", [
    ("c2_16k_gqa_outliers", 160, True), ("c2_16k_gqa_outliers", 64, False),
    ("c3_32k_llama3_8b_layer", 100, True), ("c4_128k_prefill", 44, True),
])
def test_prefill_full_size_sampled_rows(name, n_random, bf16_out):
    import gpu_util as G
    w = W.WORKLOADS[name]
    q, k, v, out, lse = _run_full(w, bf16_out)
    rows = _sample_rows(w, n_random, w.seed)
    idx = torch.from_numpy(rows).cuda()
    o_gpu = G.to_f64(out.index_select(1, idx))
    l_gpu = G.to_f64(lse.index_select(2, idx))
    _check_rows(w, q, k, v, o_gpu, l_gpu, rows, bf16_out)


@pytest.mark.parametrize("name,n_random", [
    ("c2_16k_gqa_outliers", 200), ("c3_32k_llama3_8b_layer", 80), ("c4_128k_prefill", 40),
])
def test_prefill_full_size_fp32_check_mode(name, n_random):
    """Validation mode (fp32 FMA kernels, fp32 output) at the real shapes: one seg_attn_fwd_seq
    launch over the whole workload, sampled rows -- the fixed boundary rows plus seeded random
    ones, every head -- against the oracle at max-abs 1e-4 on O and on LSE.  C2 carries the x8
    outlier key channels, C4 rows that sum 131072 weights in fp32."""
    import gpu_util as G
    import paper_2605_11744_amd as sa
    w = W.WORKLOADS[name]
    q, k, v = W.prefill_inputs(w)
    cfg = G.config_of(w, fp32_check=True)
    qd, kd, vd = G.dev_bf16(q), G.dev_bf16(k), G.dev_bf16(v)
    out = torch.full((w.batch, w.seq_len, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((w.batch, w.n_q_heads, w.seq_len), float("nan"), dtype=torch.float32, device="cuda")
    sa.seg_attn_fwd_seq(cfg, qd, kd, vd, w.seq_len, out, lse, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all()) and bool(torch.isfinite(lse).all())
    rows = _sample_rows(w, n_random, w.seed + 3)
    idx = torch.from_numpy(rows).cuda()
    o_gpu, l_gpu = G.to_f64(out.index_select(1, idx)), G.to_f64(lse.index_select(2, idx))
    o_ref, l_ref = orc.attend(q, k, v, seg_len=w.seg_len, tail_len=w.tail_len, kv_policy=w.kv_policy, rows=rows)
    eo, el = np.abs(o_gpu - o_ref), np.abs(l_gpu - l_ref)
    print(f"fp32 check mode {name}: {rows.size} rows x {w.n_q_heads} heads: |dO| max {eo.max():.3e} mean {eo.mean():.3e}, "
          f"|dLSE| max {el.max():.3e}")
    assert eo.max() <= G.FP32_MAX_ABS and el.max() <= G.FP32_MAX_ABS


def test_prefill_interleaved_policy_full_size():
    """Same FLOPs, different load balance: PAST heads spread over the KV heads (Table 11 contrasts
    contiguous and interleaved head groupings)."""
    import gpu_util as G
    w = W.interleaved(W.C2)
    assert w.kv_policy != W.C2.kv_policy
    q, k, v, out, lse = _run_full(w, True)
    rows = _sample_rows(w, 64, w.seed + 7)
    idx = torch.from_numpy(rows).cuda()
    _check_rows(w, q, k, v, G.to_f64(out.index_select(1, idx)), G.to_f64(lse.index_select(2, idx)), rows, True)


@pytest.mark.parametrize("fp32_check", [False, True])
def test_decode_c5_full_batch(fp32_check):
    """The B=64 decode workload exactly as the benchmark runs it (bf16 output), every output
    checked: cache rows written through segattn_cache_span, lengths declared, one step.  Also in
    validation mode (fp32 split-K kernels and fp32 output, windows of up to 64K rows) at 1e-4."""
    import gpu_util as G
    import paper_2605_11744_amd as sa
    w = W.C5
    S, T, D, Hkv = w.seg_len, w.tail_len, w.head_dim, w.n_kv_heads
    k_done, c_fill = W.decode_lengths(w)
    # only the rows the arena has room for are drawn (3 GB instead of 9 GB); the oracle gets zeros
    # for the rest, so a row wrongly visible or wrongly dropped on either side shows up
    q, ks, vs, _, _ = W.decode_inputs(w, k_done, c_fill, trailing_rows=G.cache_rows_held(w, k_done, c_fill))
    c = G.Cache(w, past_capacity=w.max_context, out_fp32=False, fp32_check=fp32_check)
    try:
        k_new, v_new = G.fill_cache_for_decode(c, w, ks, vs, k_done, c_fill)
        o, l = c.decode(q, k_new, v_new)
        worst = worst_l = 0.0
        for b in range(w.batch):
            n_b = int(k_done[b]) * S + int(c_fill[b])
            kf, vf = G.full_history(ks[b], vs[b], n_b, Hkv, D)
            o_ref, l_ref = orc.decode_attend(q[b], kf, vf, seg_len=S, tail_len=T, kv_policy=w.kv_policy)
            eo, el = np.abs(o[b] - o_ref), np.abs(l[b] - l_ref)
            if fp32_check:
                assert eo.max() <= G.FP32_MAX_ABS and el.max() <= G.FP32_MAX_ABS, (b, eo.max(), el.max())
            else:
                assert np.all(eo <= 1e-2 + np.abs(o_ref) * 2.0 ** -8) and eo.mean() <= 1e-3, (b, eo.max(), eo.mean())
                assert el.max() <= 1e-2 and el.mean() <= 1e-3, (b, el.max())
            worst = max(worst, eo.max())
            worst_l = max(worst_l, el.max())
        print(f"decode C5 ({'fp32 check mode' if fp32_check else 'bf16'}): worst |dO| = {worst:.3e}, worst |dLSE| = {worst_l:.3e}")
    finally:
        c.close()


@pytest.mark.parametrize("tail,long_groups", [(1024, 2), (512, 4)])
def test_whole_prompt_retrieval_mode_full_size_sampled_rows(tail, long_groups):
    """Retrieval mode on the 128K prompt as the benchmark runs it (bf16 output; R = 512, L_q = 32,
    16 anchors with 32-row windows): seg_kv_retrieve_seq chooses every segment's rows in one call,
    seg_attn_fwd_seq_retrieved attends in one launch.  With the main workload's two long-range
    groups and tail, and at the paper's operating point (Appendix F: tail 512, R = 512, half of the
    heads long-range).  Lists: sorted, distinct, inside the segment's history, and they contain the
    windows of the rows whose oracle score clearly wins; attention: sampled rows against the
    oracle with the same lists."""
    import gpu_util as G
    import paper_2605_11744_amd as sa
    w0 = W.C4
    R = 512
    policy = [2] * long_groups + [1] * (w0.n_kv_heads - long_groups)
    w = W.small("c4_retrieval", index=w0.index, seq_len=w0.seq_len, seg_len=w0.seg_len, tail_len=tail,
                n_q_heads=w0.n_q_heads, n_kv_heads=w0.n_kv_heads, head_dim=w0.head_dim, kv_policy=policy)
    params = dict(n_queries=32, pool_window=8, tail_avg=4, n_anchors=16, win_before=8, win_after=23)
    q, k, v = W.prefill_inputs(w)
    N, S, g = w.seq_len, w.seg_len, w.group
    n_seg = N // S
    cfg = G.config_of(w, out_fp32=False)
    qd, kd, vd = G.dev_bf16(q), G.dev_bf16(k), G.dev_bf16(v)
    st = torch.cuda.current_stream().cuda_stream
    r = sa.make_retrieval(**params)
    nws = sa.seg_kv_retrieve_seq_workspace_bytes(cfg, r, N)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    idx = torch.full((1, n_seg, long_groups, R), -1, dtype=torch.int32, device="cuda")
    sa.seg_kv_retrieve_seq(cfg, r, qd, kd, N, R, idx, ws, nws, st)
    nws2 = sa.seg_attn_fwd_seq_retrieved_workspace_bytes(cfg, N, R)
    ws2 = torch.empty(nws2, dtype=torch.uint8, device="cuda")
    out = torch.full((1, N, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((1, w.n_q_heads, N), float("nan"), dtype=torch.float32, device="cuda")
    sa.seg_attn_fwd_seq_retrieved(cfg, qd, kd, vd, N, idx, R, ws2, nws2, out, lse, st)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all()) and bool(torch.isfinite(lse).all())
    idx_h = idx.cpu().numpy()
    retrieved = {}
    for i in range(1, n_seg):
        for j in range(long_groups):
            lst = idx_h[0, i, j]
            assert (np.diff(lst) > 0).all() and lst[0] >= 0 and lst[-1] < i * S, (i, j)
            retrieved[(0, j, i)] = lst
    # lists of a few segments against the oracle's scores: every clearly winning row's window is in
    span = params["win_before"] + params["win_after"] + 1
    assert params["n_anchors"] * span <= R
    for i in (1, n_seg // 2, n_seg - 1):
        for j in range(long_groups):
            _, sc = orc.retrieve_indices(q[0, (i - 1) * S:i * S, j * g:(j + 1) * g], k[0, :i * S, j], R=R,
                                         return_scores=True, **params)
            nth = np.sort(sc)[-params["n_anchors"]]
            got = set(idx_h[0, i, j].tolist())
            for a_ in np.nonzero(sc > nth + 0.5)[0]:
                assert set(range(max(0, a_ - params["win_before"]), min(i * S, a_ + params["win_after"] + 1))) <= got
    rows = _sample_rows(w, 40, w.seed + 11)
    sel = torch.from_numpy(rows).cuda()
    o_ref, l_ref = orc.attend(q, k, v, seg_len=S, tail_len=tail, kv_policy=policy, rows=rows, retrieved=retrieved)
    o_gpu, l_gpu = G.to_f64(out.index_select(1, sel)), G.to_f64(lse.index_select(2, sel))
    eo, el = np.abs(o_gpu - o_ref), np.abs(l_gpu - l_ref)
    assert np.all(eo <= 1e-2 + np.abs(o_ref) * 2.0 ** -8) and eo.mean() <= 1e-3, (eo.max(), eo.mean())
    assert el.max() <= 1e-2 and el.mean() <= 1e-3, el.max()


def test_ragged_batch_full_size_sampled_rows():
    """The packed batch bench.py times (the 128K tokens of the main workload cut into 12 sequences of
    720 .. 32768 tokens, one seg_attn_fwd_varlen launch, bf16 output): rows at the start and end of
    every sequence, around its segment boundaries and at random, against the oracle run on that
    sequence alone; and everything written and finite."""
    import gpu_util as G
    w = W.C4
    lens = [32768, 24576, 20000, 16384, 12288, 8192, 6000, 4096, 3000, 2048, 1000, 720]
    assert sum(lens) == w.seq_len
    q, k, v = W.prefill_inputs(w)                       # [1, total, H, D]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cfg = G.config_of(w, out_fp32=False, batch=len(lens))
    qd, kd, vd = G.dev_bf16(q[0]), G.dev_bf16(k[0]), G.dev_bf16(v[0])
    out = torch.full((w.seq_len, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((w.n_q_heads, w.seq_len), float("nan"), dtype=torch.float32, device="cuda")
    G.sa.seg_attn_fwd_varlen(cfg, qd, kd, vd, torch.from_numpy(cu).cuda(), w.seq_len, max(lens), out, lse,
                             torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all()) and bool(torch.isfinite(lse).all())
    rng = np.random.default_rng(w.seed + 21)
    S = w.seg_len
    for b, n in enumerate(lens):
        lo = int(cu[b])
        fixed = {0, 1, 63, 64, n - 1, n - 2, n // 2, S - 1, S, S + 1, (n // S) * S - 1, (n // S) * S}
        rows = sorted({r for r in fixed if 0 <= r < n} | set(int(x) for x in rng.integers(0, n, 6)))
        rows = np.array(rows, dtype=np.int64)
        w_b = W.small(f"ragged{b}", index=0, seq_len=n, seg_len=S, tail_len=w.tail_len, n_q_heads=w.n_q_heads,
                      n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, kv_policy=list(w.kv_policy))
        idx = torch.from_numpy(rows + lo).cuda()
        o_gpu = G.to_f64(out.index_select(0, idx))[None]
        l_gpu = G.to_f64(lse.index_select(1, idx))[None]
        _check_rows(w_b, q[:, lo:lo + n], k[:, lo:lo + n], v[:, lo:lo + n], o_gpu, l_gpu, rows, True)


@pytest.mark.parametrize("kv_policy,n_kv", [([0, 1], 2), ([1, 0, 0], 3)])
def test_one_long_segment_sampled_rows(kv_policy, n_kv):
    """A single segment of 9216 rows (plain causal attention: S >= N): its K/V exceed one L2, so
    the library deals each head's query blocks to the XCDs in interleaved sub-groups (four per
    head with two heads, eight with three).  Every row written and finite, sampled rows against
    the oracle."""
    import gpu_util as G
    w = W.small("one_seg", index=150 + n_kv, seq_len=9216, seg_len=9216, tail_len=0, n_q_heads=2 * n_kv,
                n_kv_heads=n_kv, head_dim=128, kv_policy=kv_policy)
    q, k, v, out, lse = _run_full(w, bf16_out=False)
    rows = _sample_rows(w, 48, seed=151)
    idx = torch.from_numpy(rows).cuda()
    _check_rows(w, q, k, v, G.to_f64(out.index_select(1, idx)), G.to_f64(lse.index_select(2, idx)), rows, False)
