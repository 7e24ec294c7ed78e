#!/usr/bin/env python3
"""Benchmark of libsegattn on one MI355X.

A step is one pass of the whole hot path over one synthetic 128K-token prompt (B=1, 32 query
/ 8 KV heads, D=128, S=4096, T=1024, 2 of 8 KV groups with full past access):

  1. seg_attn_fwd_seq   one launch over all 32 segments (range resolution, work ordering, MFMA
                        QK^T / online softmax / PV, epilogue with LSE);
  2. seg_kv_commit_seq  the whole prompt's tail hand-off and past-pool append in one call, leaving
                        the cache exactly as segment-by-segment execution would;
  3. seg_kv_past_evict  (bookkeeping only; evicts 0 rows) and
  4. seg_attn_decode    one token on top of the 128K context (split-K + combine).

`value` = mask-useful prefill FLOPs (4*D per visible (query, key) pair; softmax work, masked
halves of diagonal tiles and skipped tiles count zero) divided by the time of the whole step,
inputs resident in HBM.  The roofline object prices the dominant kernel (the MFMA prefill
kernel) against the dense bf16 MFMA peak, from HIP-event timings of that launch alone.

Also reported on the same JSON line: the decode workload (B=64, contexts up to 64K) as
achieved HBM GB/s, segment-by-segment execution of the same prompt (bounded resident KV),
memory figures, and the fp64 oracle timed on the host cores on a bounded row sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
# HBM-side bytes of one prefill_mfma_kernel launch on the 128K workload: FETCH_SIZE + WRITE_SIZE of
# the counter runs summarised in profiles/prefill_mfma_c4_128k_hbm_traffic.txt (reads vary from run
# to run with what the long key streams find in the last-level cache): median of the three FETCH_SIZE
# runs, and (min, max) over their nine dispatches; other runs and boxes measured 7.99e9 to 10.6e9
MEASURED_TRAFFIC_BYTES = {"c4_128k_prefill": (8.93e9 + 1.09e9, (8.57e9 + 1.09e9, 9.26e9 + 1.09e9))}
NOMINAL_GFX_MHZ = 2400.0       # the clock the published peaks are quoted at


class ClockProbe:
    """Shader clock held during a timed region, from the library's clock probe: one sleeping wave per
    XCD, launched on a stream of its own just before the region, counts shader clocks against the
    device's constant-rate wall clock for `seconds` (chosen a little shorter than the region)."""

    def __init__(self, sa, torch):
        self.sa, self.started = sa, False
        self.counts = torch.zeros(2 * sa.SEGATTN_CLOCK_PROBE_WAVES, dtype=torch.int64, device="cuda")
        self.side = torch.cuda.Stream()

    def start(self, seconds):
        """Call with the device idle (the counts buffer is then cleared); returns at once."""
        us = int(seconds * 1e6)
        if 1000 <= us <= 10_000_000:
            self.khz = self.sa.segattn_clock_probe(us, self.counts, self.side.cuda_stream)
            self.started = True

    def mean_mhz(self):
        """Call after the device has been synchronized.  None if the probe did not run or its two
        counters tick at the same rate (no separate shader-clock counter)."""
        if not self.started:
            return None
        c = self.counts.cpu().numpy().reshape(-1, 2).astype(float)
        mhz = [clk / tck * self.khz / 1e3 for clk, tck in c if tck > 0 and clk > 0]
        if not mhz:
            return None
        m = sum(mhz) / len(mhz)
        return m if 300.0 < m < 3000.0 and abs(m - self.khz / 1e3) > 1.0 else None


def visible_pairs(w) -> int:
    """Closed form of the cost model (Sec. 3.5): m(m+1)/2 + m*P pairs per segment."""
    N, S, T = w.seq_len, w.seg_len, w.tail_len
    total = 0
    for pol in w.kv_policy:
        pairs = 0
        for s in range(0, N, S):
            m = min(S, N - s)
            prefix = s if pol & 2 else (min(T, s) if pol & 1 else 0)
            pairs += m * (m + 1) // 2 + m * prefix
        total += pairs * w.group
    return total * w.batch


def calibration_copy(torch):
    """Known traffic for the HBM byte counters: 1 GiB read + 1 GiB written by one copy kernel."""
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c4_128k_prefill")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the decode and streaming legs")
    ap.add_argument("--no-clock-probe", action="store_true",
                    help="run neither the clock probe beside the timed steps nor the matrix-pipe probe after them "
                         "(counter collection runs one kernel at a time: the clock probe would sleep alone and "
                         "the steps would wait for it)")
    ap.add_argument("--only", choices=("backward", "decode", "retrieve", "retrieval_seq", "rope", "ceiling", "other_configs"),
                    help="profiling aid: run just this leg (none of them needs the 128K inputs) and print it alone")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives or sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2605_11744_amd as sa
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    sa.lib()  # fails loudly if libsegattn.so has not been built
    torch.cuda.set_device(0)
    w = W.WORKLOADS[args.workload]
    if args.only:
        if args.calibration_copy:
            calibration_copy(torch)
        def retrieval_seq_only():   # random bf16 rows of the workload's shape, drawn on the GPU (timing only)
            g = torch.Generator(device="cuda").manual_seed(w.seed)
            mk = lambda h: torch.randn((w.batch, w.seq_len, h, w.head_dim), device="cuda", generator=g).to(torch.bfloat16)
            q_, k_, v_ = mk(w.n_q_heads), mk(w.n_kv_heads), mk(w.n_kv_heads)
            o_ = torch.empty_like(q_)
            return {"main": retrieval_seq_leg(sa, W, w, q_, k_, v_, o_),
                    "paper_point": retrieval_seq_leg(sa, W, w, q_, k_, v_, o_, tail=512, long_groups=4)}
        def rope_only():
            g = torch.Generator(device="cuda").manual_seed(w.seed)
            mk = lambda h: torch.randn((w.batch, w.seq_len, h, w.head_dim), device="cuda", generator=g).to(torch.bfloat16)
            return rope_leg(sa, W, w, mk(w.n_q_heads), mk(w.n_kv_heads))
        leg = {"backward": lambda: backward_leg(sa, W, w), "decode": lambda: decode_leg(sa, W),
               "retrieve": lambda: retrieve_leg(sa, W), "retrieval_seq": retrieval_seq_only, "rope": rope_only,
               "ceiling": lambda: ceiling_leg(sa, torch.zeros(1 << 28, dtype=torch.float32, device="cuda")),
               "other_configs": lambda: other_configs_leg(sa, W)}[args.only]
        print(json.dumps({args.only: leg()}))
        return 0
    N, Hq, Hkv, D, S, T = w.seq_len, w.n_q_heads, w.n_kv_heads, w.head_dim, w.seg_len, w.tail_len
    stream = torch.cuda.current_stream().cuda_stream

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    qb, kb, vb = W.prefill_inputs(w)
    q, k, v = dev(qb), dev(kb), dev(vb)
    out = torch.empty((w.batch, N, Hq, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((w.batch, Hq, N), dtype=torch.float32, device="cuda")
    cfg = sa.make_config(batch=w.batch, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, seg_len=S, tail_len=T,
                         kv_policy=w.kv_policy, past_capacity=N + S)
    arena_bytes = sa.segattn_cache_bytes(cfg)
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
    ctx = sa.segattn_create(cfg, arena, arena_bytes)
    past_heads = [h for h, p in enumerate(w.kv_policy) if p & 2]
    q1 = torch.randn((w.batch, Hq, D), device="cuda").to(torch.bfloat16)
    k1 = torch.randn((w.batch, Hkv, D), device="cuda").to(torch.bfloat16)
    v1 = torch.randn((w.batch, Hkv, D), device="cuda").to(torch.bfloat16)
    o1 = torch.empty((w.batch, Hq, D), dtype=torch.bfloat16, device="cuda")
    l1 = torch.empty((w.batch, Hq), dtype=torch.float32, device="cuda")
    ev_k0 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ev_k1 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]

    def step(i=None):
        sa.segattn_reset(ctx, stream)
        if i is not None:
            ev_k0[i].record()
        sa.seg_attn_fwd_seq(cfg, q, k, v, N, out, lse, stream)
        if i is not None:
            ev_k1[i].record()
        sa.seg_kv_commit_seq(ctx, k, v, N, stream)
        for h in past_heads[:1]:
            sa.seg_kv_past_evict(ctx, h, 0, stream)
        sa.seg_attn_decode(ctx, q1, k1, v1, o1, l1, stream)

    if args.calibration_copy:
        calibration_copy(torch)
    clock = ClockProbe(sa, torch)
    tw = time.perf_counter()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    warm_s = (time.perf_counter() - tw) / max(args.warmup, 1)
    torch.cuda.reset_peak_memory_stats()
    # the probe watches the first 70 % of the time the warm-up predicts for the timed steps, so it has
    # ended before they have; without warm-up steps there is no prediction and no probe
    if not args.no_clock_probe:
        clock.start(0.7 * warm_s * args.steps if args.warmup > 0 else 0.0)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gfx_mhz = clock.mean_mhz()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kern_ms = sum(a.elapsed_time(b) for a, b in zip(ev_k0, ev_k1)) / args.steps
    flops = 4 * D * visible_pairs(w)
    value = flops / (ms_per_step * 1e-3) / 1e12
    achieved = flops / (kern_ms * 1e-3) / 1e12
    resident = sa.segattn_resident_bytes(ctx)
    dense_kv = w.batch * Hkv * (N + 1) * D * 2 * 2
    # what the matrix pipes alone reach on this part with random operands (it is power-limited)
    pipes = None if args.no_clock_probe else mfma_probe(sa, torch, 0)

    result = {
        "metric": "segmented-attn prefill TFLOP/s (useful FLOPs) + % bf16 MFMA peak at 128K",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "seq_len": N, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": D, "seg_len": S, "tail_len": T, "kv_policy": list(w.kv_policy),
                   "step": "fwd_seq + commit_seq + evict + decode x1"},
        "pct_of_bf16_mfma_peak": round(100 * value / PEAK_BF16_TFLOPS, 2),
        "roofline": {"bound": "mfma", "kernel": "prefill_mfma_kernel", "achieved": round(achieved, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "kernel_ms": round(kern_ms, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get(w.name, (None, None))[0],
                     "traffic_range": MEASURED_TRAFFIC_BYTES.get(w.name, (None, None))[1],
                     "algorithmic_bytes": w.batch * (2 * N * Hq * D * 2 + 2 * N * Hkv * D * 2 + N * Hq * 4),
                     # the same fraction against the peak scaled to the shader clock the part held during
                     # the timed steps (the library's clock probe, mean over the XCDs); None if the probe did not run
                     "sustained_gfx_mhz": None if gfx_mhz is None else round(gfx_mhz, 1),
                     "frac_at_sustained_clock": None if gfx_mhz is None else
                     round(achieved / (PEAK_BF16_TFLOPS * gfx_mhz / NOMINAL_GFX_MHZ), 4),
                     # the matrix pipes alone, random operands, registers only: rate, clock, and this
                     # kernel as a fraction of that rate
                     "mfma_probe": pipes,
                     "frac_of_mfma_probe": None if pipes is None else round(achieved / pipes["tflops"], 4)},
        "memory": {"resident_kv_bytes_after_step": resident, "dense_causal_kv_bytes": dense_kv,
                   "ratio": round(dense_kv / resident, 3),
                   "torch_peak_allocated_bytes": int(torch.cuda.max_memory_allocated())},
    }
    sa.segattn_destroy(ctx)
    del arena

    if not args.no_extras:
        result["streaming"] = streaming_leg(sa, W, w, q, k, v, out, lse, flops)
        result["retrieval"] = retrieval_leg(sa, W, w, q, k, v, out)
        result["retrieval_seq"] = retrieval_seq_leg(sa, W, w, q, k, v, out)
        result["retrieval_seq_paper_point"] = retrieval_seq_leg(sa, W, w, q, k, v, out, tail=512, long_groups=4)
        result["ragged"] = ragged_leg(sa, W, w, q, k, v, out)
        result["rope"] = rope_leg(sa, W, w, q, k)
        result["hbm_ceilings"] = ceiling_leg(sa, q)
        del q, k, v, out, lse
        torch.cuda.empty_cache()
        result["other_configs"] = other_configs_leg(sa, W)
        result["backward"] = backward_leg(sa, W, w)
        result["decode"] = decode_leg(sa, W)
        result["retrieve"] = retrieve_leg(sa, W)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(W, w, qb, kb, vb)
    print(json.dumps(result))
    return 0


def streaming_leg(sa, W, w, q, k, v, out, lse, flops):
    """Segment-by-segment execution (seg_attn_fwd + seg_kv_commit per segment): the mode whose
    resident KV is bounded by S + T per local head plus the pool of the PAST heads."""
    import torch
    N, S = w.seq_len, w.seg_len
    cfg = sa.make_config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                         seg_len=S, tail_len=w.tail_len, kv_policy=w.kv_policy, past_capacity=N)
    nbytes = sa.segattn_cache_bytes(cfg)
    arena = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ctx = sa.segattn_create(cfg, arena, nbytes)
    stream = torch.cuda.current_stream().cuda_stream
    lse_seg = torch.empty((w.batch, w.n_q_heads, S), dtype=torch.float32, device="cuda")

    def run():
        sa.segattn_reset(ctx, stream)
        for s in range(0, N, S):
            m = min(S, N - s)
            assert w.batch == 1  # row slices of a B=1 tensor are dense
            sa.seg_attn_fwd(ctx, q[:, s:s + m], k[:, s:s + m], v[:, s:s + m], m, out[:, s:s + m], lse_seg, stream)
            sa.seg_kv_commit(ctx, k[:, s:s + m], v[:, s:s + m], m, stream)

    run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reps = 3
    for _ in range(reps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / reps
    res = {"ms": round(ms, 3), "tflops_useful": round(flops / ms / 1e9, 2),
           "resident_kv_bytes": sa.segattn_resident_bytes(ctx), "arena_bytes": nbytes}
    sa.segattn_destroy(ctx)
    return res


def retrieval_leg(sa, W, w, q, k, v, out, R=512):
    """The paper's own long-range channel on the same 128K inputs (Sec. 3.4; Appendix F: R = 512,
    L_q in [24, 64]): PAST heads see R retrieved pool rows + their segment instead of the whole
    history.  Per segment: seg_kv_retrieve (Appendix D: scores over the pool, anchors, windows),
    seg_kv_past_select (gather), seg_attn_fwd, seg_kv_commit.  Sizes the paper leaves open:
    8-row pooling windows, 4-row tail average, 16 anchors with 32-row windows."""
    import torch
    N, S, T = w.seq_len, w.seg_len, w.tail_len
    policy = [2 if (p & 2) else p for p in w.kv_policy]       # long-range heads: retrieved prefix only
    n_past = sum(1 for p in policy if p & 2)
    cfg = sa.make_config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                         seg_len=S, tail_len=T, kv_policy=policy, past_capacity=N, retrieved_capacity=R)
    nbytes = sa.segattn_cache_bytes(cfg)
    arena = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ctx = sa.segattn_create(cfg, arena, nbytes)
    stream = torch.cuda.current_stream().cuda_stream
    lse_seg = torch.empty((w.batch, w.n_q_heads, S), dtype=torch.float32, device="cuda")
    rp = sa.make_retrieval(n_queries=32, pool_window=8, tail_avg=4, n_anchors=16, win_before=8, win_after=23)
    nws = sa.seg_kv_retrieve_workspace_bytes(ctx, rp)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    idx = torch.empty((w.batch, n_past, R), dtype=torch.int32, device="cuda")
    gq = w.n_q_heads // w.n_kv_heads
    pairs = 0
    for s in range(0, N, S):
        m = min(S, N - s)
        for p in policy:
            prefix = min(R, s) if (p & 2) else (min(T, s) if (p & 1) else 0)
            pairs += gq * (m * (m + 1) // 2 + m * prefix)
    flops = 4 * w.head_dim * pairs * w.batch

    def run(with_retrieval=True):
        sa.segattn_reset(ctx, stream)
        for s in range(0, N, S):
            m = min(S, N - s)
            if s and with_retrieval:
                sa.seg_kv_retrieve(ctx, rp, q[:, s - S:s], S, R, idx, ws, nws, stream)
                sa.seg_kv_past_select(ctx, idx, R, stream)
            sa.seg_attn_fwd(ctx, q[:, s:s + m], k[:, s:s + m], v[:, s:s + m], m, out[:, s:s + m], lse_seg, stream)
            sa.seg_kv_commit(ctx, k[:, s:s + m], v[:, s:s + m], m, stream)

    def timed(flag):
        run(flag)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 3
        for _ in range(reps):
            run(flag)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / reps

    ms = timed(True)
    ms_no_prefix = timed(False)
    res = {"R": R, "kv_policy": policy, "ms": round(ms, 3), "useful_flops": flops,
           "tflops_useful": round(flops / ms / 1e9, 2),
           "ms_retrieve_and_select": round(ms - ms_no_prefix, 3),
           "resident_kv_bytes": sa.segattn_resident_bytes(ctx), "arena_bytes": nbytes}
    sa.segattn_destroy(ctx)
    return res


def retrieval_seq_leg(sa, W, w, q, k, v, out, R=512, tail=None, long_groups=None):
    """Retrieval mode for the whole 128K prompt without the per-segment host chain: one
    seg_kv_retrieve_seq (every segment's summaries scored against its pool, anchors, windows) and one
    seg_attn_fwd_seq_retrieved (gather of all retrieved prefixes, one attention launch).  Default:
    the main workload's tail and long-range groups; tail=512, long_groups=4 is the paper's operating
    point (Appendix F: M = 512, R = 512, half of the heads long-range).  Open sizes as in
    retrieval_leg."""
    import torch
    N, S = w.seq_len, w.seg_len
    T = w.tail_len if tail is None else tail
    n_long = sum(1 for p in w.kv_policy if p & 2) if long_groups is None else long_groups
    policy = [2] * n_long + [1] * (w.n_kv_heads - n_long)
    cfg = sa.make_config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                         seg_len=S, tail_len=T, kv_policy=policy)
    n_seg = (N + S - 1) // S
    rp = sa.make_retrieval(n_queries=32, pool_window=8, tail_avg=4, n_anchors=16, win_before=8, win_after=23)
    nws = sa.seg_kv_retrieve_seq_workspace_bytes(cfg, rp, N)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    nws2 = sa.seg_attn_fwd_seq_retrieved_workspace_bytes(cfg, N, R)
    ws2 = torch.empty(nws2, dtype=torch.uint8, device="cuda")
    idx = torch.empty((w.batch, n_seg, n_long, R), dtype=torch.int32, device="cuda")
    lse = torch.empty((w.batch, w.n_q_heads, N), dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    gq = w.n_q_heads // w.n_kv_heads
    pairs = 0
    for s in range(0, N, S):
        m = min(S, N - s)
        for p in policy:
            prefix = min(R, s) if (p & 2) else (min(T, s) if (p & 1) else 0)
            pairs += gq * (m * (m + 1) // 2 + m * prefix)
    flops = 4 * w.head_dim * pairs * w.batch
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

    def run(timed=False):
        if timed:
            ev[0].record()
        sa.seg_kv_retrieve_seq(cfg, rp, q, k, N, R, idx, ws, nws, st)
        if timed:
            ev[1].record()
        sa.seg_attn_fwd_seq_retrieved(cfg, q, k, v, N, idx, R, ws2, nws2, out, lse, st)
        if timed:
            ev[2].record()

    for _ in range(3):
        run()
    torch.cuda.synchronize()
    reps, t_ret, t_att = 5, 0.0, 0.0
    for _ in range(reps):
        run(True)
        torch.cuda.synchronize()
        t_ret += ev[0].elapsed_time(ev[1]) / reps
        t_att += ev[1].elapsed_time(ev[2]) / reps
    ms = t_ret + t_att
    return {"R": R, "tail_len": T, "kv_policy": policy, "ms": round(ms, 3), "ms_retrieve": round(t_ret, 3),
            "ms_gather_and_attention": round(t_att, 3), "useful_flops": flops,
            "tflops_useful": round(flops / ms / 1e9, 2), "frac_of_bf16_mfma_peak": round(flops / ms / 1e9 / PEAK_BF16_TFLOPS, 4)}


def ragged_leg(sa, W, w, q, k, v, out):
    """A packed batch of prompts of different lengths in one launch (seg_attn_fwd_varlen): the
    128K tokens of the main workload cut into 12 sequences of 2K..32K tokens (a long-context
    evaluation mix: many short prompts, a few long ones), same heads, segment and policy."""
    import torch
    lens = [32768, 24576, 20000, 16384, 12288, 8192, 6000, 4096, 3000, 2048, 1000, 720]
    assert sum(lens) == w.seq_len
    S, T = w.seg_len, w.tail_len
    gq = w.n_q_heads // w.n_kv_heads
    pairs = 0
    for n in lens:
        for s in range(0, n, S):
            m = min(S, n - s)
            for p in w.kv_policy:
                prefix = s if (p & 2) else (min(T, s) if (p & 1) else 0)
                pairs += gq * (m * (m + 1) // 2 + m * prefix)
    flops = 4 * w.head_dim * pairs
    cu = torch.tensor([0] + list(__import__("itertools").accumulate(lens)), dtype=torch.int32, device="cuda")
    cfg = sa.make_config(batch=len(lens), n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                         seg_len=S, tail_len=T, kv_policy=list(w.kv_policy))
    lse = torch.empty((w.n_q_heads, w.seq_len), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    def run():
        sa.seg_attn_fwd_varlen(cfg, q[0], k[0], v[0], cu, w.seq_len, max(lens), out[0], lse, stream)

    run()
    torch.cuda.synchronize()
    reps = 5
    t0 = time.perf_counter()
    for _ in range(reps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / reps
    return {"sequences": len(lens), "lengths": lens, "ms": round(ms, 3), "useful_flops": flops,
            "tflops_useful": round(flops / ms / 1e9, 2)}


def rope_leg(sa, W, w, q, k):
    """seg_rope_apply over the whole 128K prompt (q and k rotated in place by absolute position,
    Appendix E): every element read and written once, HBM-bound."""
    import torch
    cfg = sa.make_config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                         seg_len=w.seg_len, tail_len=w.tail_len, kv_policy=w.kv_policy, rope_theta=500000.0)
    st = torch.cuda.current_stream().cuda_stream
    sa.seg_rope_apply(cfg, q, k, w.seq_len, None, st)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 5
    e0.record()
    for _ in range(reps):
        sa.seg_rope_apply(cfg, q, k, w.seq_len, None, st)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    nbytes = 2 * (q.numel() + k.numel()) * 2
    return {"ms": round(ms, 4), "bytes": nbytes, "achieved_GBps": round(nbytes / ms / 1e6, 1),
            "frac_of_hbm_peak": round(nbytes / ms / 1e6 / PEAK_HBM_GBS, 4)}


def ceiling_leg(sa, buf):
    """What the part sustains with nothing else in the kernel.  For the access patterns of the HBM-bound
    kernels (segattn_bandwidth_probe on 1 GiB): a non-temporal read of every 16-byte piece (the
    decode and retrieval scans) and an in-place read + write of every piece (seg_rope_apply).  An even
    number of read-modify-write passes leaves the buffer as it was."""
    import torch
    nbytes = min(buf.numel() * buf.element_size(), 1 << 30)
    sink = torch.zeros(16, dtype=torch.int32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    res = {"bytes": nbytes}
    for mode, name, factor in ((0, "read_GBps", 1), (1, "read_modify_write_GBps", 2)):
        for _ in range(2):
            sa.segattn_bandwidth_probe(buf, nbytes, mode, sink, st)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        e0.record()
        for _ in range(reps):
            sa.segattn_bandwidth_probe(buf, nbytes, mode, sink, st)
        e1.record()
        torch.cuda.synchronize()
        res[name] = round(factor * nbytes / (e0.elapsed_time(e1) / reps) / 1e6, 1)
    res["mfma_random_operands"] = mfma_probe(sa, torch, 0)
    res["mfma_constant_operands"] = mfma_probe(sa, torch, 1)
    return res


def mfma_probe(sa, torch, operands):
    """The matrix pipes with nothing else busy (segattn_mfma_probe: eight independent chains of 32x32x16
    bf16 products per wave, registers only), launches about as long as the 128K prefill, with the clock
    probe beside them: the dense rate and the clock the part holds for it.  operands 0: random values
    (the switching activity of real data), 1: one constant (the part then draws less power and holds a
    higher clock: the published peak is a figure of the second kind)."""
    sink = torch.zeros(16, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    iters = 120_000
    flops = sa.segattn_mfma_probe(iters, sink, st, operands)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    sa.segattn_mfma_probe(iters, sink, st, operands)
    e1.record()
    torch.cuda.synchronize()
    one_ms = e0.elapsed_time(e1)
    clock = ClockProbe(sa, torch)
    torch.cuda.synchronize()
    reps = 3
    clock.start(0.7 * reps * one_ms * 1e-3)
    e0.record()
    for _ in range(reps):
        sa.segattn_mfma_probe(iters, sink, st, operands)
    e1.record()
    torch.cuda.synchronize()
    tflops = flops / (e0.elapsed_time(e1) / reps * 1e-3) / 1e12
    mhz = clock.mean_mhz()
    return {"tflops": round(tflops, 1), "ms_per_launch": round(e0.elapsed_time(e1) / reps, 3),
            "gfx_mhz": None if mhz is None else round(mhz, 1), "frac_of_published_peak": round(tflops / PEAK_BF16_TFLOPS, 4)}


def other_configs_leg(sa, W):
    """The other prefill configurations, one seg_attn_fwd_seq launch each on their seeded inputs
    (bf16 output), after enough launches that the clocks have come up (a 0.8 ms launch on an idle
    part runs a fifth slower)."""
    import numpy as np
    import torch
    out = {}
    for name in ("c1_2k_mha", "c2_16k_gqa_outliers", "c3_32k_llama3_8b_layer"):
        w = W.WORKLOADS[name]
        q, k, v = [torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16) for x in W.prefill_inputs(w)]
        o = torch.empty_like(q)
        lse = torch.empty((w.batch, w.n_q_heads, w.seq_len), dtype=torch.float32, device="cuda")
        cfg = sa.make_config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                             seg_len=w.seg_len, tail_len=w.tail_len, kv_policy=w.kv_policy)
        st = torch.cuda.current_stream().cuda_stream
        for _ in range(20):
            sa.seg_attn_fwd_seq(cfg, q, k, v, w.seq_len, o, lse, st)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20
        e0.record()
        for _ in range(reps):
            sa.seg_attn_fwd_seq(cfg, q, k, v, w.seq_len, o, lse, st)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        flops = 4 * w.head_dim * visible_pairs(w)
        out[name] = {"ms": round(ms, 4), "useful_flops": flops, "tflops_useful": round(flops / ms / 1e9, 1),
                     "frac_of_bf16_mfma_peak": round(flops / ms / 1e9 / PEAK_BF16_TFLOPS, 4)}
    return out


def backward_leg(sa, W, w, batch=4):
    """Training window of truncation depth K = 1 (Sec. 3.2; Appendix F: S = 4096, so 8K tokens):
    two segments per sequence with the 128K workload's heads and policy; forward once, then
    seg_attn_bwd_seq timed.  Useful FLOPs: 2D each for S, dP and dQ per visible pair plus 2D each
    for dV and dK per differentiable pair (own segment and carried tail)."""
    import torch
    S, T, D, Hq, Hkv = w.seg_len, w.tail_len, w.head_dim, w.n_q_heads, w.n_kv_heads
    n = 2 * S
    cfg = sa.make_config(batch=batch, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, seg_len=S, tail_len=T,
                         kv_policy=w.kv_policy)
    g = torch.Generator(device="cuda").manual_seed(w.seed + 7)
    mk = lambda h: torch.randn((batch, n, h, D), device="cuda", generator=g).to(torch.bfloat16)
    q, k, v, go = mk(Hq), mk(Hkv), mk(Hkv), mk(Hq)
    out, lse = torch.empty_like(q), torch.empty((batch, Hq, n), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    nws = sa.seg_attn_bwd_workspace_bytes(cfg, n)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    sa.seg_attn_fwd_seq(cfg, q, k, v, n, out, lse, st)
    run = lambda: sa.seg_attn_bwd_seq(cfg, q, k, v, out, lse, go, n, dq, dk, dv, ws, nws, st)
    for _ in range(6):   # 30 ms of work first: a 5 ms call on an idle part runs at ramping clocks
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 10
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    gq = Hq // Hkv
    vis = diff = 0
    for pol in w.kv_policy:
        for s in range(0, n, S):
            own = S * (S + 1) // 2
            tail = S * min(T, s) if pol & 1 else 0
            vis += gq * (own + (S * s if pol & 2 else tail))
            diff += gq * (own + tail)
    flops = batch * (6 * D * vis + 4 * D * diff)
    return {"workload": f"2 segments of {S} (truncation depth 1), batch {batch}, heads and policy of {w.name}",
            "ms": round(ms, 3), "useful_flops": flops, "tflops_useful": round(flops / ms / 1e9, 2),
            "frac_of_bf16_mfma_peak": round(flops / ms / 1e9 / PEAK_BF16_TFLOPS, 4)}


def retrieve_leg(sa, W):
    """Top-k retrieval operator (Appendix D) on the decode workload's caches: B = 64 sequences,
    two long-range heads each with k_b * 4096 pool rows (random bf16 rows, seeded lengths), R = 512,
    L_q = 32.  The scoring scan reads every pool K row once: HBM-bound."""
    import torch
    w = W.C5
    k_done, _ = W.decode_lengths(w)
    B, Hq, Hkv, D, S, T = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.seg_len, w.tail_len
    policy = [2 if (p & 2) else p for p in w.kv_policy]
    cfg = sa.make_config(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, seg_len=S, tail_len=T,
                         kv_policy=policy, past_capacity=w.max_context, retrieved_capacity=512)
    nbytes = sa.segattn_cache_bytes(cfg)
    arena = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(w.seed + 3)
    view = arena[: nbytes // 2 * 2].view(torch.bfloat16)
    step = 1 << 26
    for i in range(0, view.numel(), step):
        n = min(step, view.numel() - i)
        view[i:i + n] = torch.randn(n, device="cuda", generator=g, dtype=torch.float32).to(torch.bfloat16)
    ctx = sa.segattn_create(cfg, arena, nbytes)
    st = torch.cuda.current_stream().cuda_stream
    sa.seg_kv_set_lengths(ctx, [int(x) * S for x in k_done], [T] * B, [0] * B, st)
    r = sa.make_retrieval(n_queries=32, pool_window=8, tail_avg=4, n_anchors=16, win_before=8, win_after=23)
    nws = sa.seg_kv_retrieve_workspace_bytes(ctx, r)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    n_past = sum(1 for p in policy if p & 2)
    idx = torch.empty((B, n_past, 512), dtype=torch.int32, device="cuda")
    q_prev = torch.randn((B, 32, Hq, D), device="cuda", generator=g).to(torch.bfloat16)
    run = lambda: sa.seg_kv_retrieve(ctx, r, q_prev, 32, 512, idx, ws, nws, st)
    run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 10
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    k_bytes = int(sum(int(x) * S for x in k_done)) * n_past * D * 2
    sa.segattn_destroy(ctx)
    return {"workload": "pools of c5_decode_b64 (2 long-range heads), R=512, L_q=32, 16 anchors x 32-row windows",
            "ms": round(ms, 4), "k_bytes_scanned": k_bytes, "achieved_GBps": round(k_bytes / ms / 1e6, 1),
            "frac_of_hbm_peak": round(k_bytes / ms / 1e6 / PEAK_HBM_GBS, 4)}


def decode_leg(sa, W):
    """B=64 decode: contexts drawn from the seed (k_b closed segments + c_b open rows, <= 64K);
    cache rows are random bf16 written on the GPU (timing only; parity is in the tests)."""
    import torch
    w = W.C5
    k_done, c_fill = W.decode_lengths(w)
    B, Hq, Hkv, D, S, T = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.seg_len, w.tail_len
    cfg = sa.make_config(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, seg_len=S, tail_len=T,
                         kv_policy=w.kv_policy, past_capacity=w.max_context)
    nbytes = sa.segattn_cache_bytes(cfg)
    arena = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(w.seed)
    view = arena[: nbytes // 2 * 2].view(torch.bfloat16)
    step = 1 << 26
    for i in range(0, view.numel(), step):
        n = min(step, view.numel() - i)
        view[i:i + n] = torch.randn(n, device="cuda", generator=g, dtype=torch.float32).to(torch.bfloat16)
    ctx = sa.segattn_create(cfg, arena, nbytes)
    stream = torch.cuda.current_stream().cuda_stream
    q = torch.randn((B, Hq, D), device="cuda", generator=g).to(torch.bfloat16)
    kn = torch.randn((B, Hkv, D), device="cuda", generator=g).to(torch.bfloat16)
    vn = torch.randn((B, Hkv, D), device="cuda", generator=g).to(torch.bfloat16)
    out = torch.empty((B, Hq, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, Hq), dtype=torch.float32, device="cuda")
    closed = [int(x) * S for x in k_done]
    fill0 = [int(c) - 1 for c in c_fill]
    # algorithmic bytes: every K and V row the step's queries may attend to, once per KV head
    # (Eq. 13: own open segment; plus the carried tail for TAIL; plus the whole pool for PAST)
    rows = 0
    for b in range(B):
        for pol in w.kv_policy:
            closed_b = int(k_done[b]) * S
            rows += int(c_fill[b]) + (closed_b if pol & 2 else min(T, closed_b) if pol & 1 else 0)
    kv_bytes = rows * D * 2 * 2
    times = []
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for it in range(7):
        sa.seg_kv_set_lengths(ctx, closed, [T] * B, fill0, stream)
        e0.record()
        sa.seg_attn_decode(ctx, q, kn, vn, out, lse, stream)
        e1.record()
        torch.cuda.synchronize()
        if it >= 2:
            times.append(e0.elapsed_time(e1))
    ms = sum(times) / len(times)
    sa.segattn_destroy(ctx)
    return {"workload": w.name, "ms_per_step": round(ms, 4), "kv_bytes_read": kv_bytes,
            "achieved_GBps": round(kv_bytes / ms / 1e6, 1), "peak_GBps": PEAK_HBM_GBS,
            "frac_of_hbm_peak": round(kv_bytes / ms / 1e6 / PEAK_HBM_GBS, 4),
            "tokens_per_s": round(B / ms * 1e3, 1), "data": "random bf16 cache rows, seeded context lengths"}


def cpu_baseline(W, w, qb, kb, vb):
    """The fp64 oracle as it stands, on the host cores, on a bounded sample of the same
    workload: `n_rows` seeded query positions, all heads."""
    import numpy as np
    from oracle import segattn_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    rng = np.random.Generator(np.random.Philox(key=w.seed))
    n_rows = 384
    rows = np.sort(rng.choice(w.seq_len, size=n_rows, replace=False))
    t0 = time.perf_counter()
    orc.attend(qb, kb, vb, seg_len=w.seg_len, tail_len=w.tail_len, kv_policy=w.kv_policy, rows=rows)
    dt = time.perf_counter() - t0
    pairs = 0
    for pol in w.kv_policy:
        for p in rows:
            s = (int(p) // w.seg_len) * w.seg_len
            prefix = s if pol & 2 else (min(w.tail_len, s) if pol & 1 else 0)
            pairs += (int(p) - s + 1 + prefix) * w.group
    useful = 4 * w.head_dim * pairs
    return {"value": round(useful / dt / 1e12, 6), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n_rows} seeded query rows x {w.n_q_heads} heads of {w.name} "
                      f"(dense fp64 scores over all {w.seq_len} keys, explicit mask); {dt:.1f} s",
            "seconds": round(dt, 2)}


if __name__ == "__main__":
    sys.exit(main())
