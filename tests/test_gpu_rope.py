"""GPU parity of the RoPE re-indexing (Sec. 3.4, Appendix E) through the C ABI: seg_rope_apply,
and the re-rotation of a retrieved prefix inside seg_kv_past_select, against the oracle's literal
re-indexed attention (prefix keys at 0..P-1, segment queries and keys at P..P+m-1).

The library stores rotated q and k in bf16, the oracle keeps them in fp64: every rotated element
differs by up to half a bf16 ulp (2^-9 relative), which reaches the scores as noise of about
1e-3 and the outputs well inside the forward's bars."""
import numpy as np
import pytest
import torch

import paper_2605_11744_amd as sa
import workloads as W
from gpu_util import assert_parity, dev_bf16, to_f64
from oracle import segattn_oracle as orc

pytestmark = pytest.mark.gpu
THETA = 10000.0


def _rope_cfg(w, **kw):
    return sa.make_config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                          seg_len=w.seg_len, tail_len=w.tail_len, kv_policy=w.kv_policy, **kw)


@pytest.mark.parametrize("D,theta", [(64, 10000.0), (128, 500000.0)])
def test_rope_apply_matches_textbook_rotation(D, theta):
    w = W.small(seq_len=300, seg_len=128, tail_len=16, n_q_heads=4, n_kv_heads=2, head_dim=D, batch=2)
    q, k, _ = W.prefill_inputs(w)
    pos0 = [0, 70000]                                   # far positions: the angle needs double precision
    qd, kd = dev_bf16(q), dev_bf16(k)
    p0 = torch.tensor(pos0, dtype=torch.int64, device="cuda")
    sa.seg_rope_apply(_rope_cfg(w, rope_theta=theta), qd, kd, 300, p0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for got, bits in ((qd, q), (kd, k)):
        for b in range(2):
            exact = orc.rope_rotate(bits[b], pos0[b] + np.arange(300), theta)
            err = np.abs(to_f64(got[b]) - exact)
            assert (err <= 2.0 ** -8 * np.abs(exact) + 1e-5).all(), err.max()
    with pytest.raises(sa.SegattnError):                # theta missing
        sa.seg_rope_apply(_rope_cfg(w), qd, kd, 300, p0)


@pytest.mark.parametrize("fp32_check", [True, False])
def test_absolute_rotation_reproduces_reindexed_attention(fp32_check):
    n, S, T = 700, 256, 64
    w = W.small(seq_len=n, seg_len=S, tail_len=T, n_q_heads=8, n_kv_heads=4, head_dim=128,
                kv_policy=[1, 3, 0, 2], batch=1)
    q, k, v = W.prefill_inputs(w)
    cfg = _rope_cfg(w, rope_theta=THETA, fp32_check=fp32_check, out_fp32=True)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    st = torch.cuda.current_stream().cuda_stream
    sa.seg_rope_apply(cfg, qd, kd, n, None, st)
    out = torch.empty((1, n, 8, 128), dtype=torch.float32, device="cuda")
    lse = torch.empty((1, 8, n), dtype=torch.float32, device="cuda")
    sa.seg_attn_fwd_seq(cfg, qd, kd, vd, n, out, lse, st)
    torch.cuda.synchronize()
    o_ref, l_ref = orc.attend_reindexed(q, k, v, seg_len=S, tail_len=T, kv_policy=w.kv_policy, theta=THETA)
    # the rounding of the rotated operands is common to both modes: the bf16 bars apply to both
    assert_parity(to_f64(out), to_f64(lse), o_ref, l_ref, fp32_check=False, what="rope + fwd_seq")


def test_retrieved_prefix_is_rerotated_to_the_positions_before_the_segment():
    n, S, R = 640, 128, 40
    w = W.small(seq_len=n, seg_len=S, tail_len=32, n_q_heads=4, n_kv_heads=2, head_dim=128,
                kv_policy=[2, 1], batch=2)
    q, k, v = W.prefill_inputs(w)
    rng = np.random.default_rng(77)
    cfg = _rope_cfg(w, past_capacity=n, fp32_check=True, retrieved_capacity=R, rope_theta=THETA)
    nbytes = sa.segattn_cache_bytes(cfg)
    arena = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ctx = sa.segattn_create(cfg, arena, nbytes)
    st = torch.cuda.current_stream().cuda_stream
    retrieved, outs, lses = {}, [], []
    try:
        sa.segattn_reset(ctx, st)
        for i, s in enumerate(range(0, n, S)):
            if i:
                r = min(R, s)
                idx = np.stack([rng.permutation(s)[:r] for _ in range(2)]).astype(np.int32)[:, None, :]
                sa.seg_kv_past_select(ctx, torch.from_numpy(np.ascontiguousarray(idx)).cuda(), r, st)
                for b in range(2):
                    retrieved[(b, 0, i)] = idx[b, 0]
            qd, kd, vd = dev_bf16(q[:, s:s + S]), dev_bf16(k[:, s:s + S]), dev_bf16(v[:, s:s + S])
            p0 = torch.full((2,), s, dtype=torch.int64, device="cuda")
            sa.seg_rope_apply(cfg, qd, kd, S, p0, st)
            out = torch.empty((2, S, 4, 128), dtype=torch.float32, device="cuda")
            lse = torch.empty((2, 4, S), dtype=torch.float32, device="cuda")
            sa.seg_attn_fwd(ctx, qd, kd, vd, S, out, lse, st)
            sa.seg_kv_commit(ctx, kd, vd, S, st)
            torch.cuda.synchronize()
            outs.append(to_f64(out))
            lses.append(to_f64(lse))
    finally:
        sa.segattn_destroy(ctx)
    o_ref, l_ref = orc.attend_reindexed(q, k, v, seg_len=S, tail_len=32, kv_policy=w.kv_policy, theta=THETA,
                                        retrieved=retrieved)
    assert_parity(np.concatenate(outs, 1), np.concatenate(lses, 2), o_ref, l_ref, fp32_check=False,
                  what="rope + retrieval")
