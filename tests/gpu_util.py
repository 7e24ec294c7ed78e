"""Helpers for the GPU parity tests: move seeded bf16 bit patterns to the device, call the
C ABI through the Python binding, bring results back as float64 numpy arrays."""
import numpy as np
import torch

import paper_2605_11744_amd as sa

# Parity bars (bf16 MFMA path: max-abs / mean-abs; fp32 validation mode: max-abs).
BF16_MAX_ABS, BF16_MEAN_ABS, FP32_MAX_ABS = 1e-2, 1e-3, 1e-4


# Launch-shape overrides every configuration built by config_of() carries (segattn_config.
# prefill_waves / item_queues); tests switch them with monkeypatch.setitem.
TUNING = {"prefill_waves": 0, "item_queues": 0}
QUEUES_OFF, QUEUES_ON, QUEUES_ON_SMALL_GRID = 1, 2, 3


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.cuda().view(torch.bfloat16)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def config_of(w, *, fp32_check=False, out_fp32=False, past_capacity=0, batch=None, scale=0.0,
              retrieved_capacity=0):
    return sa.make_config(batch=w.batch if batch is None else batch, n_q_heads=w.n_q_heads,
                          n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, seg_len=w.seg_len,
                          tail_len=w.tail_len, kv_policy=w.kv_policy, past_capacity=past_capacity,
                          scale=scale, fp32_check=fp32_check, out_fp32=out_fp32,
                          retrieved_capacity=retrieved_capacity, **TUNING)


def fwd_seq(w, q_bits, k_bits, v_bits, *, fp32_check=False, out_fp32=True, scale=0.0):
    """One stateless launch over the whole sequence; returns (O [B,N,Hq,D], LSE [B,Hq,N]) as float64."""
    B, N = q_bits.shape[0], q_bits.shape[1]
    cfg = config_of(w, fp32_check=fp32_check, out_fp32=out_fp32, batch=B, scale=scale)
    q, k, v = dev_bf16(q_bits), dev_bf16(k_bits), dev_bf16(v_bits)
    odt = torch.float32 if (fp32_check or out_fp32) else torch.bfloat16
    out = torch.full((B, N, w.n_q_heads, w.head_dim), float("nan"), dtype=odt, device="cuda")
    lse = torch.full((B, w.n_q_heads, N), float("nan"), dtype=torch.float32, device="cuda")
    sa.seg_attn_fwd_seq(cfg, q, k, v, N, out, lse, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return to_f64(out), to_f64(lse)


def assert_parity(o_gpu, l_gpu, o_ref, l_ref, *, fp32_check, what=""):
    eo, el = np.abs(o_gpu - o_ref), np.abs(l_gpu - l_ref)
    assert np.isfinite(o_gpu).all() and np.isfinite(l_gpu).all(), f"{what}: non-finite output"
    if fp32_check:
        assert eo.max() <= FP32_MAX_ABS, f"{what}: O max-abs {eo.max():.3e}"
        assert el.max() <= FP32_MAX_ABS, f"{what}: LSE max-abs {el.max():.3e}"
    else:
        assert eo.max() <= BF16_MAX_ABS, f"{what}: O max-abs {eo.max():.3e}"
        assert el.max() <= BF16_MAX_ABS, f"{what}: LSE max-abs {el.max():.3e}"
        assert eo.mean() <= BF16_MEAN_ABS, f"{what}: O mean-abs {eo.mean():.3e}"
        assert el.mean() <= BF16_MEAN_ABS, f"{what}: LSE mean-abs {el.mean():.3e}"
    return eo.max(), eo.mean(), el.max(), el.mean()


def cache_rows_held(w, k_done, c_fill):
    """[B][Hkv]: how many trailing rows of a sequence's history the cache arena has room for when
    the token at in-segment offset c_fill - 1 is being decoded, by the layout segattn_cache_span
    documents: a PAST head's block holds every position; any other head's block holds T tail slots
    and the open segment."""
    return [[int(k_done[b]) * w.seg_len + int(c_fill[b]) if pol & 2
             else min(w.tail_len, int(k_done[b]) * w.seg_len) + int(c_fill[b])
             for pol in w.kv_policy] for b in range(w.batch)]


def fill_cache_for_decode(c, w, ks, vs, k_done, c_fill):
    """Write the rows before the token being decoded into the arena of Cache `c` through
    segattn_cache_span's layout (PAST head: row = position; other heads: tail in rows [T - tail, T),
    open segment from row T) and declare the lengths.  ks[b][h], vs[b][h] hold trailing rows of the
    history (at least as many as cache_rows_held), newest last.  Returns (k_new, v_new) [B,Hkv,D]."""
    S, T, D, Hkv = w.seg_len, w.tail_len, w.head_dim, w.n_kv_heads
    k_new = np.zeros((w.batch, Hkv, D), dtype=np.uint16)
    v_new = np.zeros((w.batch, Hkv, D), dtype=np.uint16)
    held = cache_rows_held(w, k_done, c_fill)
    for b in range(w.batch):
        for h, pol in enumerate(w.kv_policy):
            kk, vv = ks[b][h][-held[b][h]:], vs[b][h][-held[b][h]:]
            k_new[b, h], v_new[b, h] = kk[-1], vv[-1]
            kd, vd = c.rows_view(b, h)
            n_prev = kk.shape[0] - 1
            first = 0 if pol & 2 else T - min(T, int(k_done[b]) * S)
            if n_prev:
                kd[first:first + n_prev] = dev_bf16(kk[:-1])
                vd[first:first + n_prev] = dev_bf16(vv[:-1])
    sa.seg_kv_set_lengths(c.ctx, [int(x) * S for x in k_done], [min(T, int(x) * S) for x in k_done],
                          [int(x) - 1 for x in c_fill], c.stream)
    return k_new, v_new


def full_history(ks_b, vs_b, n_b, Hkv, D):
    """[n_b, Hkv, D] float64 K and V of one sequence for the oracle: rows that were not drawn
    (older than a head's trailing rows) are zero."""
    from oracle import segattn_oracle as orc
    kf, vf = np.zeros((n_b, Hkv, D)), np.zeros((n_b, Hkv, D))
    for h in range(Hkv):
        kept = ks_b[h].shape[0]
        kf[n_b - kept:, h] = orc.widen(ks_b[h])
        vf[n_b - kept:, h] = orc.widen(vs_b[h])
    return kf, vf


class Cache:
    """A context over a torch-allocated arena."""

    def __init__(self, w, *, past_capacity, fp32_check=False, out_fp32=True, batch=None, scale=0.0,
                 retrieved_capacity=0):
        self.w = w
        self.B = w.batch if batch is None else batch
        self.cfg = config_of(w, fp32_check=fp32_check, out_fp32=out_fp32, past_capacity=past_capacity,
                             batch=self.B, scale=scale, retrieved_capacity=retrieved_capacity)
        self.odt = torch.float32 if (fp32_check or out_fp32) else torch.bfloat16
        self.bytes = sa.segattn_cache_bytes(self.cfg)
        assert self.bytes > 0
        self.arena = torch.empty(self.bytes, dtype=torch.uint8, device="cuda")
        self.ctx = sa.segattn_create(self.cfg, self.arena, self.bytes)
        self.stream = torch.cuda.current_stream().cuda_stream
        sa.segattn_reset(self.ctx, self.stream)

    def close(self):
        if self.ctx:
            torch.cuda.synchronize()
            sa.segattn_destroy(self.ctx)
            self.ctx = None

    def fwd(self, q_bits, k_bits, v_bits):
        m = q_bits.shape[1]
        q, k, v = dev_bf16(q_bits), dev_bf16(k_bits), dev_bf16(v_bits)
        out = torch.full((self.B, m, self.w.n_q_heads, self.w.head_dim), float("nan"), dtype=self.odt, device="cuda")
        lse = torch.full((self.B, self.w.n_q_heads, m), float("nan"), dtype=torch.float32, device="cuda")
        sa.seg_attn_fwd(self.ctx, q, k, v, m, out, lse, self.stream)
        sa.seg_kv_commit(self.ctx, k, v, m, self.stream)
        torch.cuda.synchronize()
        return to_f64(out), to_f64(lse)

    def select(self, idx):
        """idx: integer array [B, n_past, R] of pool rows; becomes the retrieved prefix."""
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        t = torch.from_numpy(idx).cuda()
        sa.seg_kv_past_select(self.ctx, t, idx.shape[2], self.stream)
        torch.cuda.synchronize()

    def decode(self, q_bits, k_bits, v_bits):
        q, k, v = dev_bf16(q_bits), dev_bf16(k_bits), dev_bf16(v_bits)
        out = torch.full((self.B, self.w.n_q_heads, self.w.head_dim), float("nan"), dtype=self.odt, device="cuda")
        lse = torch.full((self.B, self.w.n_q_heads), float("nan"), dtype=torch.float32, device="cuda")
        sa.seg_attn_decode(self.ctx, q, k, v, out, lse, self.stream)
        torch.cuda.synchronize()
        return to_f64(out), to_f64(lse)

    def rows_view(self, b, kv_head):
        """(K, V) views [cap, D] (bf16) of the arena block of (b, kv_head)."""
        k_off, v_off, cap = sa.segattn_cache_span(self.ctx, b, kv_head)
        D = self.w.head_dim
        kv = self.arena[k_off:k_off + cap * D * 2].view(torch.bfloat16).view(cap, D)
        vv = self.arena[v_off:v_off + cap * D * 2].view(torch.bfloat16).view(cap, D)
        return kv, vv
