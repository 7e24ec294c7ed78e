"""GPU checks of retrieval mode for a whole prompt, stateless (Sec. 3.4 "Long-Range Channel"; Eq. 13,
second case; Appendix D): seg_kv_retrieve_seq chooses every segment's R pool rows in one call,
seg_attn_fwd_seq_retrieved attends to [retrieved rows ; own segment] in one launch, both through
the C ABI.  Index lists: exact against the oracle where the best scores tower over the rest
(planted keys), valid (sorted, distinct, inside the segment's history) everywhere.  Attention:
the oracle's attend() with the same lists, element by element."""
import numpy as np
import pytest
import torch

import paper_2605_11744_amd as sa
import workloads as W
from gpu_util import assert_parity, config_of, dev_bf16, to_f64
from oracle import segattn_oracle as orc

pytestmark = pytest.mark.gpu
PARAMS = dict(n_queries=24, pool_window=8, tail_avg=4, n_anchors=4, win_before=2, win_after=5)


def _bits(x):
    return W.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def retrieve_seq(cfg, params, qd, kd, n, R, B, n_seg, n_past):
    r = sa.make_retrieval(**params)
    nws = sa.seg_kv_retrieve_seq_workspace_bytes(cfg, r, n)
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    idx = torch.full((B, n_seg, n_past, R), -1, dtype=torch.int32, device="cuda")
    sa.seg_kv_retrieve_seq(cfg, r, qd, kd, n, R, idx, ws, nws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return idx


def fwd_retrieved(cfg, qd, kd, vd, n, idx, R, Hq, D):
    B = qd.shape[0]
    nws = sa.seg_attn_fwd_seq_retrieved_workspace_bytes(cfg, n, R)
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    out = torch.full((B, n, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, Hq, n), float("nan"), dtype=torch.float32, device="cuda")
    sa.seg_attn_fwd_seq_retrieved(cfg, qd, kd, vd, n, idx, R, ws, nws, out, lse, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return to_f64(out), to_f64(lse)


def _planted_prompt(seed, n, S, D, g, B, policy):
    """Random prompt whose last 24 query rows of every segment are one constant vector per head (so
    every summary of a head is that vector) and in which a few keys of long-range head 0 are large
    multiples of query head 0's vector: their scores tower over the rest in every later segment."""
    rng = np.random.default_rng(seed)
    w = W.small("planted_seq", index=400 + seed, seq_len=n, seg_len=S, tail_len=16, n_q_heads=len(policy) * g,
                n_kv_heads=len(policy), head_dim=D, kv_policy=policy, batch=B)
    q, k, v = W.prefill_inputs(w)
    u = _bits(rng.standard_normal((B, len(policy) * g, D)))
    for s in range(0, n, S):
        e = min(s + S, n)
        q[:, max(s, e - 24):e] = u[:, None]
    kv0 = [h for h, pol in enumerate(policy) if pol & 2][0]
    uf = orc.widen(u[:, kv0 * g])                          # first query head of the first long-range group
    for b in range(B):
        rows = rng.choice(n - S, size=6, replace=False)
        for j, r in enumerate(rows):
            k[b, r, kv0] = _bits((40.0 - 4.0 * j) * uf[b] / np.linalg.norm(uf[b]))
    return w, q, k, v


@pytest.mark.parametrize("D,g,R,n,S", [(128, 2, 48, 900, 128), (64, 4, 30, 1024, 256), (128, 4, 128, 1500, 128)])
def test_whole_prompt_retrieval_gives_the_oracle_lists_on_planted_rows(D, g, R, n, S):
    B, policy = 2, [2, 1, 2]
    w, q, k, v = _planted_prompt(D + g, n, S, D, g, B, policy)
    cfg = config_of(w, fp32_check=True)
    n_seg = (n + S - 1) // S
    idx = retrieve_seq(cfg, PARAMS, dev_bf16(q), dev_bf16(k), n, R, B, n_seg, 2).cpu().numpy()
    past_heads = [0, 2]
    for b in range(B):
        for i in range(1, n_seg):
            for j, h in enumerate(past_heads):
                got = idx[b, i, j]
                assert (np.diff(got) > 0).all() and got[0] >= 0 and got[-1] < i * S, (b, i, h)
                if h == 0:        # the planted head: the list is decided by clear margins
                    want = orc.retrieve_indices(q[b, (i - 1) * S:i * S, h * g:(h + 1) * g], k[b, :i * S, h], R=R, **PARAMS)
                    assert list(got) == list(want), (b, i)


@pytest.mark.parametrize("fp32_check", [True, False])
@pytest.mark.parametrize("D,g,R,n,S,policy", [
    (128, 4, 48, 700, 128, [1, 2, 0, 2]),      # ragged last segment, every policy a retrieval-mode layer has
    (64, 2, 100, 640, 128, [2, 1]),
    (128, 1, 5, 521, 100, [2, 2, 1]),          # tiny prefix, segment length not a multiple of the tiles
])
def test_retrieve_then_attend_matches_oracle(fp32_check, D, g, R, n, S, policy):
    B = 2
    w = W.small("ret_seq", index=410, seq_len=n, seg_len=S, tail_len=32, n_q_heads=len(policy) * g,
                n_kv_heads=len(policy), head_dim=D, kv_policy=policy, batch=B)
    q, k, v = W.prefill_inputs(w)
    cfg = config_of(w, fp32_check=fp32_check, out_fp32=True)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    n_seg = (n + S - 1) // S
    past_heads = [h for h, pol in enumerate(policy) if pol & 2]
    idx = retrieve_seq(cfg, PARAMS, qd, kd, n, R, B, n_seg, len(past_heads))
    o, l = fwd_retrieved(cfg, qd, kd, vd, n, idx, R, w.n_q_heads, D)
    idx_h = idx.cpu().numpy()
    retrieved = {(b, h, i): idx_h[b, i, j] for b in range(B) for i in range(1, n_seg) for j, h in enumerate(past_heads)}
    for key, lst in retrieved.items():
        assert len(set(lst.tolist())) == R and lst.min() >= 0 and lst.max() < key[2] * S
    o_ref, l_ref = orc.attend(q, k, v, seg_len=S, tail_len=32, kv_policy=policy, retrieved=retrieved)
    assert_parity(o, l, o_ref, l_ref, fp32_check=fp32_check, what=f"retrieved prefixes D={D} R={R}")


def test_callers_own_lists_in_any_order_and_full_lists_equal_full_history():
    """The lists need not come from the operator and their order is irrelevant (softmax over a set);
    lists that name the whole history reproduce what seg_attn_fwd_seq computes for a PAST head."""
    n, S, B, D = 512, 128, 2, 128
    w = W.small("ret_own", index=411, seq_len=n, seg_len=S, tail_len=32, n_q_heads=4, n_kv_heads=2, head_dim=D,
                kv_policy=[2, 1], batch=B)
    q, k, v = W.prefill_inputs(w)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    cfg = config_of(w, fp32_check=True)
    rng = np.random.default_rng(5)
    R = 50
    idx = np.zeros((B, 4, 1, R), dtype=np.int32)
    retrieved = {}
    for b in range(B):
        for i in range(1, 4):
            idx[b, i, 0] = rng.permutation(i * S)[:R]
            retrieved[(b, 0, i)] = idx[b, i, 0]
    o, l = fwd_retrieved(cfg, qd, kd, vd, n, torch.from_numpy(idx).cuda(), R, 4, D)
    o_ref, l_ref = orc.attend(q, k, v, seg_len=S, tail_len=32, kv_policy=[2, 1], retrieved=retrieved)
    assert_parity(o, l, o_ref, l_ref, fp32_check=True, what="caller's lists")
    # R = S: every row of the first segment's history for segment 1 -> equals the full-history result there
    full = np.zeros((B, 4, 1, S), dtype=np.int32)
    full[:, :, 0] = np.arange(S)
    o2, l2 = fwd_retrieved(cfg, qd, kd, vd, n, torch.from_numpy(full).cuda(), S, 4, D)
    out = torch.empty((B, n, 4, D), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, 4, n), dtype=torch.float32, device="cuda")
    sa.seg_attn_fwd_seq(cfg, qd, kd, vd, n, out, lse, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    np.testing.assert_allclose(o2[:, S:2 * S], to_f64(out)[:, S:2 * S], atol=2e-6)
    np.testing.assert_allclose(l2[:, :, S:2 * S], to_f64(lse)[:, :, S:2 * S], atol=2e-5)


def test_retrieved_prefixes_are_rerotated_to_the_positions_before_their_segments():
    """With rope_theta the gathered keys, stored at their absolute positions, are turned to the R
    positions just before the segment (Appendix E up to a common shift): the oracle's literal
    re-indexed attention with the same lists."""
    theta = 10000.0
    n, S, R, B = 640, 128, 40, 2
    w = W.small("ret_rope", index=412, seq_len=n, seg_len=S, tail_len=32, n_q_heads=4, n_kv_heads=2, head_dim=128,
                kv_policy=[2, 1], batch=B)
    q, k, v = W.prefill_inputs(w)
    cfg = sa.make_config(batch=B, n_q_heads=4, n_kv_heads=2, head_dim=128, seg_len=S, tail_len=32, kv_policy=[2, 1],
                         fp32_check=True, rope_theta=theta)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    sa.seg_rope_apply(cfg, qd, kd, n, None, torch.cuda.current_stream().cuda_stream)
    rng = np.random.default_rng(78)
    idx = np.zeros((B, 5, 1, R), dtype=np.int32)
    retrieved = {}
    for b in range(B):
        for i in range(1, 5):
            idx[b, i, 0] = rng.permutation(i * S)[:R]
            retrieved[(b, 0, i)] = idx[b, i, 0]
    o, l = fwd_retrieved(cfg, qd, kd, vd, n, torch.from_numpy(idx).cuda(), R, 4, 128)
    o_ref, l_ref = orc.attend_reindexed(q, k, v, seg_len=S, tail_len=32, kv_policy=[2, 1], theta=theta, retrieved=retrieved)
    # rotated operands are stored in bf16: the bf16 bars apply (as for every RoPE parity test)
    assert_parity(o, l, o_ref, l_ref, fp32_check=False, what="rope + retrieved prefixes")


def test_validation_of_the_whole_prompt_calls():
    w = W.small("ret_val", index=413, seq_len=256, seg_len=128, tail_len=16, n_q_heads=8, n_kv_heads=2, head_dim=64,
                kv_policy=[2, 1])
    r = sa.make_retrieval(**PARAMS)
    cfg = config_of(w)
    assert sa.seg_kv_retrieve_seq_workspace_bytes(cfg, r, 256) > 0
    assert sa.seg_attn_fwd_seq_retrieved_workspace_bytes(cfg, 256, 129) == 0                     # R > S
    assert sa.seg_attn_fwd_seq_retrieved_workspace_bytes(config_of(w.with_policy([3, 1])), 256, 8) == 0  # TAIL|PAST
    assert sa.seg_kv_retrieve_seq_workspace_bytes(config_of(w.with_policy([1, 1])), r, 256) == 0  # no PAST head
    assert sa.seg_kv_retrieve_seq_workspace_bytes(cfg, sa.make_retrieval(**{**PARAMS, "n_anchors": 33}), 256) == 0
    with pytest.raises(sa.SegattnError) as e:
        sa.seg_kv_retrieve_seq(cfg, r, 256, 256, 256, 8, 256, 256, 16)                           # workspace too small
    assert e.value.status == sa.SEGATTN_EINVAL
    with pytest.raises(sa.SegattnError) as e:
        sa.seg_attn_fwd_seq_retrieved(cfg, 256, 256, 256, 256, 0, 8, 256, 1 << 30, 256, 256)     # null lists
    assert e.value.status == sa.SEGATTN_EINVAL
