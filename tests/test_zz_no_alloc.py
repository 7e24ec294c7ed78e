"""seg_attn_bwd_seq_static -- the backward pass for callers that cannot allocate (code under graph
capture, tight loops, harnesses that forbid hipMalloc) -- against seg_attn_bwd_seq through the
C ABI: same inputs, the row statistic in the library's built-in scratch array instead of a
caller's workspace.  Two calls in a row, the second on a smaller problem (the array keeps the
first call's contents), and the size limit."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _both_ways(w, fp32_check=False):
    import gpu_util as G
    import paper_2605_11744_amd as sa
    B, N = w.batch, w.seq_len
    q, k, v = W.prefill_inputs(w)
    go = W.grad_inputs(w)
    cfg = G.config_of(w, fp32_check=fp32_check, out_fp32=True)
    qd, kd, vd, gd = G.dev_bf16(q), G.dev_bf16(k), G.dev_bf16(v), G.dev_bf16(go)
    out = torch.empty((B, N, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, w.n_q_heads, N), dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    sa.seg_attn_fwd_seq(cfg, qd, kd, vd, N, out, lse, st)

    def grads():
        dq = torch.full_like(out, float("nan"))
        dk = torch.full((B, N, w.n_kv_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        return dq, dk, torch.full_like(dk, float("nan"))

    ref = grads()
    nws = sa.seg_attn_bwd_workspace_bytes(cfg, N)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    sa.seg_attn_bwd_seq(cfg, qd, kd, vd, out, lse, gd, N, *ref, ws, nws, st)
    got = grads()                       # every buffer exists before the call: it must allocate nothing
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    sa.seg_attn_bwd_seq_static(cfg, qd, kd, vd, out, lse, gd, N, *got, st)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return got, ref


def _assert_same(got, ref, what):
    for name, g_, r_ in zip(("dQ", "dK", "dV"), got, ref):
        assert bool(torch.isfinite(g_).all()), f"{what}: {name} not finite"
        err = (g_.double() - r_.double()).abs()
        G_ = max(1.0, float(r_.abs().max()))
        # the bar of the backward parity tests, relative to the largest gradient of the tensor ...
        assert float(err.max()) <= 1e-2 * G_ and float(err.mean()) <= 1e-3 * G_, f"{what}: {name} {float(err.max()):.3e}"
        # ... and in fact the same kernels on the same inputs: nothing may differ at all
        assert torch.equal(g_, r_), f"{what}: {name} differs from seg_attn_bwd_seq by {float(err.max()):.3e}"


def test_static_scratch_backward_matches_workspace_backward_twice_in_a_row():
    big = W.small("noalloc_a", index=180, seq_len=1500, seg_len=512, tail_len=128, n_q_heads=16, n_kv_heads=4,
                  head_dim=128, kv_policy=[3, 1, 0, 2], batch=2)
    small = W.small("noalloc_b", index=181, seq_len=333, seg_len=100, tail_len=37, n_q_heads=8, n_kv_heads=4,
                    head_dim=64, kv_policy=[1, 3, 2, 0], batch=1)
    _assert_same(*_both_ways(big), "first call")
    _assert_same(*_both_ways(small), "second, smaller call")       # scratch still holds the first call's values
    _assert_same(*_both_ways(small, fp32_check=True), "validation mode")


def test_static_scratch_backward_rejects_what_does_not_fit():
    import gpu_util as G
    import paper_2605_11744_amd as sa
    w = W.small("noalloc_c", index=182, seq_len=64, seg_len=32, tail_len=8, n_q_heads=32, n_kv_heads=8, head_dim=128,
                kv_policy=[1] * 8, batch=4)
    cfg = G.config_of(w)
    n_fit = sa.SEGATTN_BWD_STATIC_SCRATCH_BYTES // (2 * 4 * 32 * 4)        # 8192 rows: exactly the array
    for n, status in ((n_fit + 1, sa.SEGATTN_ESCRATCH), (1 << 22, sa.SEGATTN_ESCRATCH), (0, sa.SEGATTN_EINVAL)):
        with pytest.raises(sa.SegattnError) as e:                           # refused before any pointer is used
            sa.seg_attn_bwd_seq_static(cfg, 256, 256, 256, 256, 256, 256, n, 256, 256, 256)
        assert e.value.status == status
    assert "scratch" in sa.strerror(sa.SEGATTN_ESCRATCH)
