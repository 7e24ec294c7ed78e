"""ctypes binding of libsegattn's C ABI (include/segattn.h): same names, argument
marshalling only.  Device buffers are passed as torch tensors (their data_ptr()) or raw
integer addresses; nothing here computes anything."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libsegattn.so")

SEGATTN_OK, SEGATTN_EINVAL, SEGATTN_ECAPACITY, SEGATTN_ESTATE, SEGATTN_EHIP, SEGATTN_ESCRATCH = range(6)
SEGATTN_BWD_STATIC_SCRATCH_BYTES = 8 << 20
SEGATTN_SEG, SEGATTN_TAIL, SEGATTN_PAST = 0, 1, 2


class SegattnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class segattn_config(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("seg_len", ctypes.c_int32), ("tail_len", ctypes.c_int32),
        ("past_capacity", ctypes.c_int64), ("kv_policy", ctypes.POINTER(ctypes.c_uint8)),
        ("scale", ctypes.c_float), ("fp32_check", ctypes.c_int32), ("out_fp32", ctypes.c_int32),
        ("retrieved_capacity", ctypes.c_int32), ("rope_theta", ctypes.c_float),
        ("prefill_waves", ctypes.c_int32), ("item_queues", ctypes.c_int32),
    ]


class segattn_retrieval(ctypes.Structure):
    _fields_ = [("n_queries", ctypes.c_int32), ("pool_window", ctypes.c_int32), ("tail_avg", ctypes.c_int32),
                ("n_anchors", ctypes.c_int32), ("win_before", ctypes.c_int32), ("win_after", ctypes.c_int32)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libsegattn.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2605_11744_amd.build` "
                "(hipcc, gfx950); libsegattn has no CPU or PyTorch fallback")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        cfgp = ctypes.POINTER(segattn_config)
        sig = {
            "segattn_cache_bytes": (sz, [cfgp]),
            "segattn_create": (ctypes.c_int, [cfgp, vp, sz, ctypes.POINTER(vp)]),
            "segattn_destroy": (None, [vp]),
            "segattn_reset": (ctypes.c_int, [vp, vp]),
            "seg_attn_fwd": (ctypes.c_int, [vp, vp, vp, vp, i32, vp, vp, vp]),
            "seg_attn_fwd_seq": (ctypes.c_int, [cfgp, vp, vp, vp, i64, vp, vp, vp]),
            "seg_attn_fwd_varlen": (ctypes.c_int, [cfgp, vp, vp, vp, vp, i64, i64, vp, vp, vp]),
            "segattn_layer_policy": (ctypes.c_int, [i32, ctypes.POINTER(i32), i32, i32, ctypes.POINTER(ctypes.c_uint8)]),
            "seg_rope_apply": (ctypes.c_int, [cfgp, vp, vp, i64, vp, vp]),
            "seg_attn_bwd_workspace_bytes": (sz, [cfgp, i64]),
            "seg_attn_bwd_seq": (ctypes.c_int, [cfgp, vp, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp, sz, vp]),
            "seg_attn_bwd_seq_static": (ctypes.c_int, [cfgp, vp, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp]),
            "seg_attn_bwd_varlen_workspace_bytes": (sz, [cfgp, i64]),
            "seg_attn_bwd_varlen": (ctypes.c_int, [cfgp, vp, vp, vp, vp, vp, vp, vp, i64, i64, vp, vp, vp, vp, sz, vp]),
            "seg_kv_commit": (ctypes.c_int, [vp, vp, vp, i32, vp]),
            "seg_kv_commit_seq": (ctypes.c_int, [vp, vp, vp, i64, vp]),
            "seg_kv_past_append": (ctypes.c_int, [vp, i32, vp, vp, i64, vp]),
            "seg_kv_past_select": (ctypes.c_int, [vp, vp, i32, vp]),
            "seg_kv_past_evict": (ctypes.c_int, [vp, i32, i64, vp]),
            "seg_kv_past_keep_recent": (ctypes.c_int, [vp, i32, i64, vp]),
            "seg_kv_retrieve_workspace_bytes": (sz, [vp, ctypes.POINTER(segattn_retrieval)]),
            "seg_kv_retrieve": (ctypes.c_int, [vp, ctypes.POINTER(segattn_retrieval), vp, i32, i32, vp, vp, sz, vp]),
            "seg_kv_retrieve_seq_workspace_bytes": (sz, [cfgp, ctypes.POINTER(segattn_retrieval), i64]),
            "seg_kv_retrieve_seq": (ctypes.c_int, [cfgp, ctypes.POINTER(segattn_retrieval), vp, vp, i64, i32, vp, vp, sz, vp]),
            "seg_attn_fwd_seq_retrieved_workspace_bytes": (sz, [cfgp, i64, i32]),
            "seg_attn_fwd_seq_retrieved": (ctypes.c_int, [cfgp, vp, vp, vp, i64, vp, i32, vp, sz, vp, vp, vp]),
            "seg_kv_lengths": (ctypes.c_int, [vp, ctypes.POINTER(i64), ctypes.POINTER(i32), ctypes.POINTER(i32)]),
            "seg_kv_set_lengths": (ctypes.c_int, [vp, ctypes.POINTER(i64), ctypes.POINTER(i32), ctypes.POINTER(i32), vp]),
            "segattn_cache_span": (ctypes.c_int, [vp, i32, i32, ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(i64)]),
            "segattn_resident_bytes": (sz, [vp]),
            "seg_attn_decode": (ctypes.c_int, [vp, vp, vp, vp, vp, vp, vp]),
            "segattn_bandwidth_probe": (ctypes.c_int, [vp, sz, i32, vp, vp]),
            "segattn_clock_probe": (ctypes.c_int, [ctypes.c_uint32, vp, ctypes.POINTER(i32), vp]),
            "segattn_mfma_probe": (ctypes.c_int, [i32, i32, vp, ctypes.POINTER(i64), vp]),
            "segattn_strerror": (ctypes.c_char_p, [ctypes.c_int]),
            "segattn_version": (ctypes.c_char_p, []),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


EXPORTS = ("segattn_cache_bytes", "segattn_create", "segattn_destroy", "segattn_reset", "seg_attn_fwd",
           "seg_attn_fwd_seq", "seg_attn_fwd_varlen", "segattn_layer_policy", "seg_rope_apply", "seg_attn_bwd_workspace_bytes", "seg_attn_bwd_seq", "seg_attn_bwd_seq_static", "seg_attn_bwd_varlen_workspace_bytes", "seg_attn_bwd_varlen", "seg_kv_commit", "seg_kv_commit_seq", "seg_kv_past_append", "seg_kv_past_select", "seg_kv_retrieve_workspace_bytes", "seg_kv_retrieve", "seg_kv_retrieve_seq_workspace_bytes", "seg_kv_retrieve_seq", "seg_attn_fwd_seq_retrieved_workspace_bytes", "seg_attn_fwd_seq_retrieved", "seg_kv_past_evict", "seg_kv_past_keep_recent",
           "seg_kv_lengths", "seg_kv_set_lengths", "segattn_cache_span", "segattn_resident_bytes",
           "seg_attn_decode", "segattn_bandwidth_probe", "segattn_clock_probe", "segattn_mfma_probe", "segattn_strerror", "segattn_version")


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def _check(st: int, where: str) -> None:
    if st != SEGATTN_OK:
        raise SegattnError(st, where)


def make_config(*, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, seg_len: int,
                tail_len: int, kv_policy: Sequence[int], past_capacity: int = 0, scale: float = 0.0,
                fp32_check: bool = False, out_fp32: bool = False,
                retrieved_capacity: int = 0, rope_theta: float = 0.0, prefill_waves: int = 0,
                item_queues: int = 0) -> segattn_config:
    pol = (ctypes.c_uint8 * len(kv_policy))(*[int(p) for p in kv_policy])
    cfg = segattn_config(batch, n_q_heads, n_kv_heads, head_dim, seg_len, tail_len, past_capacity,
                         ctypes.cast(pol, ctypes.POINTER(ctypes.c_uint8)), scale,
                         int(fp32_check), int(out_fp32), int(retrieved_capacity), float(rope_theta),
                         int(prefill_waves), int(item_queues))
    cfg._policy_keepalive = pol
    return cfg


def strerror(status: int) -> str:
    return lib().segattn_strerror(int(status)).decode()


def segattn_version() -> str:
    return lib().segattn_version().decode()


def segattn_cache_bytes(cfg: segattn_config) -> int:
    return int(lib().segattn_cache_bytes(ctypes.byref(cfg)))


def segattn_create(cfg: segattn_config, cache, cache_bytes: int) -> int:
    ctx = ctypes.c_void_p()
    _check(lib().segattn_create(ctypes.byref(cfg), _ptr(cache), cache_bytes, ctypes.byref(ctx)), "segattn_create")
    return ctx.value


def segattn_destroy(ctx: int) -> None:
    lib().segattn_destroy(ctx)


def segattn_reset(ctx: int, stream=None) -> None:
    _check(lib().segattn_reset(ctx, _ptr(stream)), "segattn_reset")


def seg_attn_fwd(ctx: int, q, k, v, m: int, out, lse, stream=None) -> None:
    _check(lib().seg_attn_fwd(ctx, _ptr(q), _ptr(k), _ptr(v), m, _ptr(out), _ptr(lse), _ptr(stream)), "seg_attn_fwd")


def seg_attn_fwd_seq(cfg: segattn_config, q, k, v, n: int, out, lse, stream=None) -> None:
    _check(lib().seg_attn_fwd_seq(ctypes.byref(cfg), _ptr(q), _ptr(k), _ptr(v), n, _ptr(out), _ptr(lse),
                                  _ptr(stream)), "seg_attn_fwd_seq")


def seg_attn_fwd_varlen(cfg: segattn_config, q, k, v, cu_seqlens, total: int, max_seqlen: int, out, lse,
                        stream=None) -> None:
    _check(lib().seg_attn_fwd_varlen(ctypes.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), total,
                                     max_seqlen, _ptr(out), _ptr(lse), _ptr(stream)), "seg_attn_fwd_varlen")


def segattn_layer_policy(n_kv_heads: int, long_heads: Sequence[int], layer_in_l_long: bool):
    lh = (ctypes.c_int32 * max(1, len(long_heads)))(*[int(h) for h in long_heads])
    out = (ctypes.c_uint8 * n_kv_heads)()
    _check(lib().segattn_layer_policy(n_kv_heads, lh, len(long_heads), int(bool(layer_in_l_long)), out),
           "segattn_layer_policy")
    return list(out)


def seg_rope_apply(cfg: segattn_config, q, k, rows: int, pos0=None, stream=None) -> None:
    _check(lib().seg_rope_apply(ctypes.byref(cfg), _ptr(q), _ptr(k), rows, _ptr(pos0), _ptr(stream)), "seg_rope_apply")


def seg_attn_bwd_workspace_bytes(cfg: segattn_config, n: int) -> int:
    return int(lib().seg_attn_bwd_workspace_bytes(ctypes.byref(cfg), n))


def seg_attn_bwd_seq(cfg: segattn_config, q, k, v, out, lse, dout, n: int, dq, dk, dv, workspace,
                     workspace_bytes: int, stream=None) -> None:
    _check(lib().seg_attn_bwd_seq(ctypes.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dout), n,
                                  _ptr(dq), _ptr(dk), _ptr(dv), _ptr(workspace), workspace_bytes, _ptr(stream)),
           "seg_attn_bwd_seq")


def seg_attn_bwd_seq_static(cfg: segattn_config, q, k, v, out, lse, dout, n: int, dq, dk, dv, stream=None) -> None:
    _check(lib().seg_attn_bwd_seq_static(ctypes.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse),
                                         _ptr(dout), n, _ptr(dq), _ptr(dk), _ptr(dv), _ptr(stream)),
           "seg_attn_bwd_seq_static")


def seg_attn_bwd_varlen_workspace_bytes(cfg: segattn_config, total: int) -> int:
    return int(lib().seg_attn_bwd_varlen_workspace_bytes(ctypes.byref(cfg), total))


def seg_attn_bwd_varlen(cfg: segattn_config, q, k, v, out, lse, dout, cu_seqlens, total: int, max_seqlen: int,
                        dq, dk, dv, workspace, workspace_bytes: int, stream=None) -> None:
    _check(lib().seg_attn_bwd_varlen(ctypes.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dout),
                                     _ptr(cu_seqlens), total, max_seqlen, _ptr(dq), _ptr(dk), _ptr(dv),
                                     _ptr(workspace), workspace_bytes, _ptr(stream)), "seg_attn_bwd_varlen")


def seg_kv_commit(ctx: int, k, v, m: int, stream=None) -> None:
    _check(lib().seg_kv_commit(ctx, _ptr(k), _ptr(v), m, _ptr(stream)), "seg_kv_commit")


def seg_kv_commit_seq(ctx: int, k, v, n: int, stream=None) -> None:
    _check(lib().seg_kv_commit_seq(ctx, _ptr(k), _ptr(v), n, _ptr(stream)), "seg_kv_commit_seq")


def seg_kv_past_append(ctx: int, kv_head: int, k, v, rows: int, stream=None) -> None:
    _check(lib().seg_kv_past_append(ctx, kv_head, _ptr(k), _ptr(v), rows, _ptr(stream)), "seg_kv_past_append")


def seg_kv_past_select(ctx: int, idx, R: int, stream=None) -> None:
    _check(lib().seg_kv_past_select(ctx, _ptr(idx), R, _ptr(stream)), "seg_kv_past_select")


def make_retrieval(*, n_queries: int, pool_window: int, tail_avg: int, n_anchors: int, win_before: int,
                   win_after: int) -> segattn_retrieval:
    return segattn_retrieval(n_queries, pool_window, tail_avg, n_anchors, win_before, win_after)


def seg_kv_retrieve_workspace_bytes(ctx: int, r: segattn_retrieval) -> int:
    return int(lib().seg_kv_retrieve_workspace_bytes(ctx, ctypes.byref(r)))


def seg_kv_retrieve(ctx: int, r: segattn_retrieval, q_prev, m: int, R: int, idx_out, workspace,
                    workspace_bytes: int, stream=None) -> None:
    _check(lib().seg_kv_retrieve(ctx, ctypes.byref(r), _ptr(q_prev), m, R, _ptr(idx_out), _ptr(workspace),
                                 workspace_bytes, _ptr(stream)), "seg_kv_retrieve")


def seg_kv_retrieve_seq_workspace_bytes(cfg: segattn_config, r: segattn_retrieval, n: int) -> int:
    return int(lib().seg_kv_retrieve_seq_workspace_bytes(ctypes.byref(cfg), ctypes.byref(r), n))


def seg_kv_retrieve_seq(cfg: segattn_config, r: segattn_retrieval, q, k, n: int, R: int, idx_out, workspace,
                        workspace_bytes: int, stream=None) -> None:
    _check(lib().seg_kv_retrieve_seq(ctypes.byref(cfg), ctypes.byref(r), _ptr(q), _ptr(k), n, R, _ptr(idx_out),
                                     _ptr(workspace), workspace_bytes, _ptr(stream)), "seg_kv_retrieve_seq")


def seg_attn_fwd_seq_retrieved_workspace_bytes(cfg: segattn_config, n: int, R: int) -> int:
    return int(lib().seg_attn_fwd_seq_retrieved_workspace_bytes(ctypes.byref(cfg), n, R))


def seg_attn_fwd_seq_retrieved(cfg: segattn_config, q, k, v, n: int, idx, R: int, workspace, workspace_bytes: int,
                               out, lse, stream=None) -> None:
    _check(lib().seg_attn_fwd_seq_retrieved(ctypes.byref(cfg), _ptr(q), _ptr(k), _ptr(v), n, _ptr(idx), R,
                                            _ptr(workspace), workspace_bytes, _ptr(out), _ptr(lse), _ptr(stream)),
           "seg_attn_fwd_seq_retrieved")


def seg_kv_past_evict(ctx: int, kv_head: int, n_oldest: int, stream=None) -> None:
    _check(lib().seg_kv_past_evict(ctx, kv_head, n_oldest, _ptr(stream)), "seg_kv_past_evict")


def seg_kv_past_keep_recent(ctx: int, kv_head: int, max_rows: int, stream=None) -> None:
    _check(lib().seg_kv_past_keep_recent(ctx, kv_head, max_rows, _ptr(stream)), "seg_kv_past_keep_recent")


def seg_kv_lengths(ctx: int, batch: int, n_kv_heads: int):
    past = (ctypes.c_int64 * (batch * n_kv_heads))()
    tail = (ctypes.c_int32 * batch)()
    fill = (ctypes.c_int32 * batch)()
    _check(lib().seg_kv_lengths(ctx, past, tail, fill), "seg_kv_lengths")
    return ([list(past[b * n_kv_heads:(b + 1) * n_kv_heads]) for b in range(batch)], list(tail), list(fill))


def seg_kv_set_lengths(ctx: int, closed_rows: Sequence[int], tail: Sequence[int], seg_fill: Sequence[int],
                       stream=None) -> None:
    n = len(closed_rows)
    _check(lib().seg_kv_set_lengths(ctx, (ctypes.c_int64 * n)(*[int(x) for x in closed_rows]),
                                    (ctypes.c_int32 * n)(*[int(x) for x in tail]),
                                    (ctypes.c_int32 * n)(*[int(x) for x in seg_fill]), _ptr(stream)),
           "seg_kv_set_lengths")


def segattn_cache_span(ctx: int, b: int, kv_head: int):
    k_off, v_off, cap = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_int64()
    _check(lib().segattn_cache_span(ctx, b, kv_head, ctypes.byref(k_off), ctypes.byref(v_off), ctypes.byref(cap)),
           "segattn_cache_span")
    return k_off.value, v_off.value, cap.value


def segattn_resident_bytes(ctx: int) -> int:
    return int(lib().segattn_resident_bytes(ctx))


def segattn_bandwidth_probe(buf, nbytes: int, mode: int, sink, stream=None) -> None:
    _check(lib().segattn_bandwidth_probe(_ptr(buf), nbytes, mode, _ptr(sink), _ptr(stream)), "segattn_bandwidth_probe")


SEGATTN_CLOCK_PROBE_WAVES = 8


def segattn_clock_probe(microseconds: int, counts, stream=None) -> int:
    """Launches the clock probe; returns the wall clock's rate in kHz.  counts: device, 16 uint64."""
    khz = ctypes.c_int32(0)
    _check(lib().segattn_clock_probe(microseconds, _ptr(counts), ctypes.byref(khz), _ptr(stream)), "segattn_clock_probe")
    return int(khz.value)


def segattn_mfma_probe(iterations: int, sink, stream=None, operands: int = 0) -> int:
    """Launches the matrix-pipe probe (operands 0: random values, 1: one constant); returns the
    floating-point operations of the launch."""
    flops = ctypes.c_int64(0)
    _check(lib().segattn_mfma_probe(iterations, operands, _ptr(sink), ctypes.byref(flops), _ptr(stream)),
           "segattn_mfma_probe")
    return int(flops.value)


def seg_attn_decode(ctx: int, q, k_new, v_new, out, lse, stream=None) -> None:
    _check(lib().seg_attn_decode(ctx, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), _ptr(lse), _ptr(stream)),
           "seg_attn_decode")
