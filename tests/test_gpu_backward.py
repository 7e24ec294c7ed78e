"""GPU parity of the backward pass (training with truncated backpropagation over segments,
Sec. 3.2): seg_attn_fwd_seq then seg_attn_bwd_seq through the C ABI against the fp64 oracle's
attend_backward on the same seeded inputs.

Tolerance.  fp32 check mode: max-abs 1e-4 like the forward.  bf16 MFMA mode: P and dS are rounded
to bf16 (relative 2^-9) before the second products and accumulated in fp32, so the error of a
gradient element is a few 2^-9 of the magnitude of the sums it is made of; the bar is the
forward's (max-abs 1e-2, mean-abs 1e-3) relative to G = max(1, max |gradient|) of the tensor."""
import numpy as np
import pytest
import torch

import paper_2605_11744_amd as sa
import workloads as W
from gpu_util import config_of, dev_bf16, to_f64
from oracle import segattn_oracle as orc

pytestmark = pytest.mark.gpu


def run_backward(w, q, k, v, go, *, fp32_check, out_fp32=True):
    B, N = q.shape[0], q.shape[1]
    cfg = config_of(w, fp32_check=fp32_check, out_fp32=out_fp32, batch=B)
    wide = fp32_check or out_fp32
    qd, kd, vd, gd = dev_bf16(q), dev_bf16(k), dev_bf16(v), dev_bf16(go)
    odt = torch.float32 if wide else torch.bfloat16
    out = torch.empty((B, N, w.n_q_heads, w.head_dim), dtype=odt, device="cuda")
    lse = torch.empty((B, w.n_q_heads, N), dtype=torch.float32, device="cuda")
    dq = torch.full_like(out, float("nan"))
    dk = torch.full((B, N, w.n_kv_heads, w.head_dim), float("nan"), dtype=odt, device="cuda")
    dv = torch.full_like(dk, float("nan"))
    nws = sa.seg_attn_bwd_workspace_bytes(cfg, N)
    assert nws >= B * w.n_q_heads * N * 4
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    sa.seg_attn_fwd_seq(cfg, qd, kd, vd, N, out, lse, st)
    sa.seg_attn_bwd_seq(cfg, qd, kd, vd, out, lse, gd, N, dq, dk, dv, ws, nws, st)
    torch.cuda.synchronize()
    return to_f64(dq), to_f64(dk), to_f64(dv)


def assert_grad_parity(got, ref, *, fp32_check, what):
    for name, g_, r_ in zip(("dQ", "dK", "dV"), got, ref):
        assert np.isfinite(g_).all(), f"{what}: {name} not finite"
        err = np.abs(g_ - r_)
        G = max(1.0, float(np.abs(r_).max()))
        if fp32_check:
            assert err.max() <= 1e-4 * G, f"{what}: {name} max-abs {err.max():.3e} (G={G:.2f})"
        else:
            assert err.max() <= 1e-2 * G, f"{what}: {name} max-abs {err.max():.3e} (G={G:.2f})"
            assert err.mean() <= 1e-3 * G, f"{what}: {name} mean-abs {err.mean():.3e} (G={G:.2f})"


CASES = [
    # D, Hq, Hkv, S, T, n, policy, batch
    (64, 4, 4, 128, 32, 512, [1, 3, 0, 2], 1),      # every policy, whole segments
    (128, 8, 2, 256, 64, 700, [1, 3], 2),           # GQA 4:1, ragged last segment, two sequences
    (128, 4, 2, 96, 96, 330, [1, 2], 1),            # T = S, segment not a multiple of the tiles
    (64, 2, 1, 1024, 100, 777, [1], 1),             # a single short segment (S > n)
    (128, 2, 2, 37, 5, 150, [3, 1], 1),             # tiny segments, tail inside one tile
]


@pytest.mark.parametrize("fp32_check", [True, False, "queued"])
@pytest.mark.parametrize("D,Hq,Hkv,S,T,n,policy,batch", CASES)
def test_backward_matches_oracle(fp32_check, D, Hq, Hkv, S, T, n, policy, batch, monkeypatch):
    if fp32_check == "queued":   # the MFMA kernels, dQ (and the forward) as a resident grid that takes
        fp32_check = False       # its work items from queues (what large launches do by themselves)
        import gpu_util
        monkeypatch.setitem(gpu_util.TUNING, "item_queues", gpu_util.QUEUES_ON_SMALL_GRID)
    w = W.small(seq_len=n, seg_len=S, tail_len=T, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D,
                kv_policy=policy, batch=batch)
    q, k, v = W.prefill_inputs(w)
    go = W.grad_inputs(w)
    got = run_backward(w, q, k, v, go, fp32_check=fp32_check)
    ref = orc.attend_backward(q, k, v, go, seg_len=S, tail_len=T, kv_policy=policy)
    assert_grad_parity(got, ref, fp32_check=fp32_check, what=f"bwd D={D} S={S} T={T} n={n}")


def test_backward_two_segment_window_in_bf16_outputs():
    """The training window of truncation depth 1 (two segments) with bf16 forward output and bf16
    gradients, the configuration the benchmark times."""
    S, T, n = 512, 128, 1024
    w = W.small(seq_len=n, seg_len=S, tail_len=T, n_q_heads=8, n_kv_heads=2, head_dim=128,
                kv_policy=[3, 1], batch=2)
    q, k, v = W.prefill_inputs(w)
    go = W.grad_inputs(w)
    got = run_backward(w, q, k, v, go, fp32_check=False, out_fp32=False)
    ref = orc.attend_backward(q, k, v, go, seg_len=S, tail_len=T, kv_policy=w.kv_policy)
    for name, g_, r_ in zip(("dQ", "dK", "dV"), got, ref):
        err = np.abs(g_ - r_)
        G = max(1.0, float(np.abs(r_).max()))
        # bf16 storage of the result adds up to 2^-9 relative per element
        assert err.max() <= 2e-2 * G and err.mean() <= 2e-3 * G, f"{name}: {err.max():.3e} {err.mean():.3e} G={G:.2f}"


_WINDOW_REF = {}


@pytest.mark.parametrize("out_fp32", [False, True])
def test_backward_training_window_at_benchmark_shape(out_fp32):
    """The 8K training window of truncation depth 1 at the shape the benchmark times (two segments
    of 4096, tail 1024, 32 query / 8 KV heads of width 128, two PAST groups), one sequence, launched
    as the library chooses (dQ as a resident grid on the item queues, dK/dV longest blocks first
    with the rotating assignment): every element of dQ, dK, dV against the oracle.  With bf16
    results (the benchmark's configuration) the forward output that feeds delta and the three
    gradients are stored in bf16, which adds half a bf16 spacing (2^-8 relative) per element."""
    S, T, n = 4096, 1024, 8192
    w = W.small("tbptt1_window", index=160, seq_len=n, seg_len=S, tail_len=T, n_q_heads=32, n_kv_heads=8,
                head_dim=128, kv_policy=list(W.C4.kv_policy))
    q, k, v = W.prefill_inputs(w)
    go = W.grad_inputs(w)
    got = run_backward(w, q, k, v, go, fp32_check=False, out_fp32=out_fp32)
    if "ref" not in _WINDOW_REF:   # about a minute of fp64 on the host cores: once for both result types
        _WINDOW_REF["ref"] = orc.attend_backward(q, k, v, go, seg_len=S, tail_len=T, kv_policy=w.kv_policy)
    ref = _WINDOW_REF["ref"]
    for name, g_, r_ in zip(("dQ", "dK", "dV"), got, ref):
        assert np.isfinite(g_).all(), f"{name} not finite"
        err = np.abs(g_ - r_)
        G = max(1.0, float(np.abs(r_).max()))
        print(f"backward 2x4096 ({'fp32' if out_fp32 else 'bf16'} results) {name}: max-abs {err.max():.3e} "
              f"mean-abs {err.mean():.3e}, max |gradient| {G:.2f}")
        slack = 0.0 if out_fp32 else np.abs(r_) * 2.0 ** -8
        assert np.all(err <= 1e-2 * G + slack), f"{name}: max-abs {err.max():.3e} (G={G:.2f})"
        assert err.mean() <= 1e-3 * G, f"{name}: mean-abs {err.mean():.3e} (G={G:.2f})"


def test_backward_validates_arguments():
    w = W.small(seq_len=64, seg_len=32, tail_len=8, n_q_heads=2, n_kv_heads=2, head_dim=64, kv_policy=[1, 1])
    cfg = config_of(w)
    with pytest.raises(sa.SegattnError) as e:
        sa.seg_attn_bwd_seq(cfg, 256, 256, 256, 256, 256, 256, 64, 256, 256, 256, 256, 16)   # workspace too small
    assert e.value.status == sa.SEGATTN_EINVAL
    with pytest.raises(sa.SegattnError) as e:
        sa.seg_attn_bwd_seq(cfg, 256, 256, 256, 256, 256, 0, 64, 256, 256, 256, 256, 1 << 20)  # null dout
    assert e.value.status == sa.SEGATTN_EINVAL


@pytest.mark.parametrize("fp32_check", [True, False])
@pytest.mark.parametrize("D,Hq,Hkv,policy", [(128, 8, 2, [1, 3]), (64, 4, 4, [1, 3, 0, 2])])
def test_packed_ragged_backward_matches_oracle(fp32_check, D, Hq, Hkv, policy):
    """seg_attn_fwd_varlen then seg_attn_bwd_varlen on sequences of different lengths packed without
    padding (an empty one, a one-token one, one ending a row past a segment boundary) against the
    oracle's per-sequence backward."""
    lens = [300, 1, 0, 257, 128, 77]
    S, T = 128, 32
    total = sum(lens)
    w = W.small("ragged_bwd", index=150, seq_len=total, seg_len=S, tail_len=T, n_q_heads=Hq, n_kv_heads=Hkv,
                head_dim=D, kv_policy=policy)
    q, k, v = W.prefill_inputs(w)
    go = W.grad_inputs(w)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cfg = config_of(w, fp32_check=fp32_check, out_fp32=True, batch=len(lens))
    qd, kd, vd, gd = dev_bf16(q[0]), dev_bf16(k[0]), dev_bf16(v[0]), dev_bf16(go[0])
    cud = torch.from_numpy(cu).cuda()
    out = torch.empty((total, Hq, D), dtype=torch.float32, device="cuda")
    lse = torch.empty((Hq, total), dtype=torch.float32, device="cuda")
    dq = torch.full_like(out, float("nan"))
    dk = torch.full((total, Hkv, D), float("nan"), dtype=torch.float32, device="cuda")
    dv = torch.full_like(dk, float("nan"))
    nws = sa.seg_attn_bwd_varlen_workspace_bytes(cfg, total)
    assert nws >= Hq * total * 4
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    sa.seg_attn_fwd_varlen(cfg, qd, kd, vd, cud, total, max(lens), out, lse, st)
    sa.seg_attn_bwd_varlen(cfg, qd, kd, vd, out, lse, gd, cud, total, max(lens), dq, dk, dv, ws, nws, st)
    torch.cuda.synchronize()
    ref = orc.attend_backward_packed(q[0], k[0], v[0], go[0], cu, seg_len=S, tail_len=T, kv_policy=policy)
    assert_grad_parity((to_f64(dq), to_f64(dk), to_f64(dv)), ref, fp32_check=fp32_check, what="packed backward")
