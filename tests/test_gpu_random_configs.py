"""GPU parity on seeded random small configurations: segment and tail lengths that are not
multiples of the 32-key step, tails longer than a step, one-row segments, every GQA ratio the
kernels specialise on, both head dimensions, both workgroup shapes, dense and packed batches,
forward and backward.  The oracle is the judge in every case."""
import numpy as np
import pytest
import torch

import paper_2605_11744_amd as sa
import workloads as W
from gpu_util import config_of, dev_bf16, to_f64, assert_parity
from oracle import segattn_oracle as orc

pytestmark = pytest.mark.gpu


def _configs(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        D = int(rng.choice([64, 128]))
        Hkv = int(rng.choice([1, 2, 3, 4]))
        g = int(rng.choice([1, 2, 3, 4, 8]))
        S = int(rng.choice([1, 7, 31, 32, 33, 64, 95, 128, 200, 257]))
        T = int(rng.integers(0, S + 1))
        n_seq = int(rng.integers(1, 4))
        lens = [int(rng.integers(1, 3 * S + 40)) for _ in range(n_seq)]
        policy = [int(rng.integers(0, 4)) for _ in range(Hkv)]
        out.append(dict(D=D, Hkv=Hkv, g=g, S=S, T=T, lens=lens, policy=policy, idx=400 + i))
    return out


CONFIGS = _configs(28, 20260511)


@pytest.mark.parametrize("waves", ["4", "8"])
@pytest.mark.parametrize("c", CONFIGS, ids=lambda c: f"D{c['D']}g{c['g']}kv{c['Hkv']}S{c['S']}T{c['T']}n{'-'.join(map(str, c['lens']))}")
def test_random_config_forward_and_backward(c, waves, monkeypatch):
    if c["D"] != 128 and waves == "4":
        pytest.skip("the wave count only exists in the head_dim-128 MFMA kernel")
    import gpu_util
    monkeypatch.setitem(gpu_util.TUNING, "prefill_waves", int(waves))
    D, Hkv, g, S, T, lens, policy = c["D"], c["Hkv"], c["g"], c["S"], c["T"], c["lens"], c["policy"]
    Hq = Hkv * g
    total = sum(lens)
    w = W.small("rnd", index=c["idx"], seq_len=total, seg_len=S, tail_len=T, n_q_heads=Hq, n_kv_heads=Hkv,
                head_dim=D, kv_policy=policy)
    q, k, v = W.prefill_inputs(w)
    go = W.grad_inputs(w)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cfg = config_of(w, out_fp32=True, batch=len(lens))
    qd, kd, vd, gd = dev_bf16(q[0]), dev_bf16(k[0]), dev_bf16(v[0]), dev_bf16(go[0])
    cud = torch.from_numpy(cu).cuda()
    out = torch.full((total, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((Hq, total), float("nan"), dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    sa.seg_attn_fwd_varlen(cfg, qd, kd, vd, cud, total, max(lens), out, lse, st)
    torch.cuda.synchronize()
    kw = dict(seg_len=S, tail_len=T, kv_policy=policy)
    o_ref, l_ref = orc.attend_packed(q[0], k[0], v[0], cu, **kw)
    assert_parity(to_f64(out), to_f64(lse), o_ref, l_ref, fp32_check=False, what="forward")
    if waves == "8":  # the backward kernels do not depend on the forward's workgroup shape
        dq = torch.full_like(out, float("nan"))
        dk = torch.full((total, Hkv, D), float("nan"), dtype=torch.float32, device="cuda")
        dv = torch.full_like(dk, float("nan"))
        nws = sa.seg_attn_bwd_varlen_workspace_bytes(cfg, total)
        ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
        sa.seg_attn_bwd_varlen(cfg, qd, kd, vd, out, lse, gd, cud, total, max(lens), dq, dk, dv, ws, nws, st)
        torch.cuda.synchronize()
        ref = orc.attend_backward_packed(q[0], k[0], v[0], go[0], cu, **kw)
        for name, g_, r_ in zip(("dQ", "dK", "dV"), (to_f64(dq), to_f64(dk), to_f64(dv)), ref):
            assert np.isfinite(g_).all(), f"{name} not finite"
            err = np.abs(g_ - r_)
            G = max(1.0, float(np.abs(r_).max()))
            assert err.max() <= 1e-2 * G and err.mean() <= 1e-3 * G, f"{name}: max {err.max():.3e} mean {err.mean():.3e} G={G:.2f}"


def _stateful_configs(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        long_prefix = i % 4 == 3   # every fourth: prefixes of thousands of rows (the library splits them)
        D = 128 if long_prefix else int(rng.choice([64, 128]))
        Hkv = int(rng.choice([1, 2, 4]))
        g = int(rng.choice([1, 2, 3, 4, 8])) if not long_prefix else int(rng.choice([1, 2, 4]))
        S = int(rng.choice([512, 700, 1024])) if long_prefix else int(rng.choice([7, 32, 33, 64, 95, 128, 200]))
        T = int(rng.integers(0, min(S, 300) + 1))
        B = int(rng.integers(1, 4)) if not long_prefix else int(rng.integers(1, 3))
        n_pre = int(rng.integers(3 * S, 6 * S)) if long_prefix else int(rng.integers(1, 4 * S + 20))
        n_dec = int(rng.integers(1, 6))
        policy = [int(rng.integers(0, 4)) for _ in range(Hkv)]
        if long_prefix and not any(p & 2 for p in policy):
            policy[0] |= 2
        chunks = [int(rng.integers(1, S + 1)) for _ in range(5)]
        out.append(dict(D=D, Hkv=Hkv, g=g, S=S, T=T, B=B, n_pre=n_pre, n_dec=n_dec, policy=policy, chunks=chunks,
                        idx=500 + i))
    return out


@pytest.mark.parametrize("c", _stateful_configs(16, 20260512),
                         ids=lambda c: f"D{c['D']}g{c['g']}kv{c['Hkv']}S{c['S']}T{c['T']}B{c['B']}n{c['n_pre']}+{c['n_dec']}")
def test_random_config_streaming_then_decode(c, monkeypatch):
    """Segment-by-segment prefill in random chunks (the library's own choice of workgroup shape and
    of prefix pieces), then a few decode steps: every output row against the oracle's row of the
    full sequence."""
    from gpu_util import Cache
    D, Hkv, g, S, T, B = c["D"], c["Hkv"], c["g"], c["S"], c["T"], c["B"]
    n_pre, n_dec, policy, chunks = c["n_pre"], c["n_dec"], c["policy"], c["chunks"]
    N = n_pre + n_dec
    w = W.small("rnd_state", index=c["idx"], seq_len=N, seg_len=S, tail_len=T, n_q_heads=Hkv * g, n_kv_heads=Hkv,
                head_dim=D, kv_policy=policy, batch=B)
    q, k, v = W.prefill_inputs(w)
    o_ref, l_ref = orc.attend(q, k, v, seg_len=S, tail_len=T, kv_policy=policy)
    cache = Cache(w, past_capacity=((N + S) // S) * S)
    try:
        o = np.zeros_like(o_ref)
        l = np.zeros_like(l_ref)
        pos, i = 0, 0
        while pos < n_pre:
            m = min(chunks[i % len(chunks)], S - pos % S, n_pre - pos)
            i += 1
            oc, lc = cache.fwd(q[:, pos:pos + m], k[:, pos:pos + m], v[:, pos:pos + m])
            o[:, pos:pos + m] = oc
            l[:, :, pos:pos + m] = lc
            pos += m
        for p_ in range(n_pre, N):
            od, ld = cache.decode(q[:, p_], k[:, p_], v[:, p_])
            o[:, p_] = od
            l[:, :, p_] = ld
        assert_parity(o, l, o_ref, l_ref, fp32_check=False, what="streaming + decode")
    finally:
        cache.close()
