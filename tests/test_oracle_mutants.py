"""The pins must be sharp: a plausible mistake planted anywhere in the oracle (on the CPU,
in a private copy of its source) has to make at least one pin fail."""
import os
import types

import pytest

import test_oracle_pins as pins
from conftest import ROOT

SRC = open(os.path.join(ROOT, "oracle", "segattn_oracle.py")).read()

MUTANTS = {
    "causal_excludes_diagonal": ("vis = (j >= s) & (j <= p)", "vis = (j >= s) & (j < p) | (j == s)"),
    "causal_sees_one_ahead": ("(j <= p)", "(j <= p + 1)"),
    "tail_one_row_short": ("(j >= max(0, s - tail_len)) & (j < s)", "(j >= max(0, s - tail_len + 1)) & (j < s)"),
    "tail_one_row_long": ("(j >= max(0, s - tail_len)) & (j < s)", "(j >= max(0, s - tail_len - 1)) & (j < s)"),
    "tail_from_two_segments_back": ("(j >= max(0, s - tail_len)) & (j < s)",
                                    "(j >= max(0, s - seg_len - tail_len)) & (j < s - seg_len + tail_len)"),
    "past_ignores_policy_bit": ("if policy & POLICY_PAST:", "if policy & POLICY_TAIL:"),
    "past_includes_future": ("vis |= (j >= evicted) & (j < s)", "vis |= (j >= evicted)"),
    "eviction_ignored": ("vis |= (j >= evicted) & (j < s)", "vis |= (j < s)"),
    "segment_start_off_by_one": ("s = (p // seg_len) * seg_len", "s = ((p + 1) // seg_len) * seg_len"),
    "scale_dropped": ("@ kb.T) * scale", "@ kb.T)"),
    "scale_is_inverse_d": ("1.0 / np.sqrt(D)", "1.0 / D"),
    "head_map_modulo": ("for h in range(kvh * g, (kvh + 1) * g):", "for h in range(kvh, Hq, Hkv):"),
    "values_from_keys": ("pr @ vb", "pr @ kb"),
    "lse_without_max": ("(zmax + np.log(denom))", "(np.log(denom))"),
    "lse_base_2": ("np.log(denom)", "np.log2(denom)"),
    "no_normalisation": ("pr = e / denom", "pr = e"),
    "mask_added_as_zero": ("np.where(mask, z, -np.inf)", "np.where(mask, z, 0.0)"),
    "decode_uses_previous_row": ("rows=[n - 1], evicted=evicted", "rows=[max(n - 2, 0)], evicted=evicted"),
    "bf16_widen_shift": ("<< np.uint32(16)", "<< np.uint32(15)"),
    "retrieved_list_ignored": ("            vis[idx] = True\n", "            pass\n"),
    "retrieved_added_to_whole_history": ("        if retrieved is None:                      # forward-only", "        if True:                      # forward-only"),
    "retrieved_of_previous_segment": ("retrieved.get((b, kvh, int(p) // seg_len), ())", "retrieved.get((b, kvh, int(p) // seg_len - 1), ())"),
    "retrieved_of_first_sequence_for_all": ("retrieved.get((b, kvh, int(p) // seg_len), ())", "retrieved.get((0, kvh, int(p) // seg_len), ())"),
    "retrieved_duplicates_accepted": ("if np.unique(idx).size != idx.size:", "if False:"),
    "decode_retrieved_of_next_segment": ("{(0, h, (n - 1) // seg_len): idx", "{(0, h, n // seg_len): idx"),
    "bwd_gradient_into_past_rows": ("dk[b, :, kvh, :] += scale * ((ds * grad).T @ q[b, rr, h, :])", "dk[b, :, kvh, :] += scale * ((ds * mask).T @ q[b, rr, h, :])"),
    "bwd_value_gradient_into_past_rows": ("(pr * grad).T @ dout[b, rr, h, :]", "(pr * mask).T @ dout[b, rr, h, :]"),
    "bwd_tail_not_differentiable": ("        diff |= (j >= max(0, s - tail_len)) & (j < s)", "        pass"),
    "bwd_delta_dropped": ("ds = pr * (dp - delta)", "ds = pr * dp"),
    "bwd_dq_scale_dropped": ("dq[b, rr, h, :] = scale * (ds @ kb)", "dq[b, rr, h, :] = (ds @ kb)"),
    "bwd_dk_uses_dout": ("((ds * grad).T @ q[b, rr, h, :])", "((ds * grad).T @ dout[b, rr, h, :])"),
    "bwd_dp_from_keys": ("dp = dout[b, rr, h, :] @ vb.T", "dp = dout[b, rr, h, :] @ kb.T"),
    "bwd_group_heads_overwrite": ("dv[b, :, kvh, :] += (pr * grad)", "dv[b, :, kvh, :] = (pr * grad)"),
    "rope_interleaved_pairs_sign": ("np.concatenate([a * cos - b * sin, a * sin + b * cos], axis=-1)", "np.concatenate([a * cos + b * sin, -a * sin + b * cos], axis=-1)"),
    "rope_frequency_exponent": ("* 2.0 / D)", "* 1.0 / D)"),
    "reindex_segment_starts_at_zero": ("ks = rope_rotate(k[b, s:s + m, kvh:kvh + 1, :], P + np.arange(m), theta)[:, 0]", "ks = rope_rotate(k[b, s:s + m, kvh:kvh + 1, :], np.arange(m), theta)[:, 0]"),
    "reindex_queries_not_shifted": ("qs = rope_rotate(q[b, s:s + m, h:h + 1, :], P + np.arange(m), theta)[:, 0]", "qs = rope_rotate(q[b, s:s + m, h:h + 1, :], np.arange(m), theta)[:, 0]"),
    "reindex_values_rotated": ("vc = np.concatenate([v[b, pref, kvh, :], v[b, s:s + m, kvh, :]])", "vc = np.concatenate([rope_rotate(v[b, pref, kvh:kvh + 1, :], np.arange(P), theta)[:, 0], v[b, s:s + m, kvh, :]])"),
    "retrieval_tail_average_missing": ("    out.append(last[L - min(int(tail_avg), L):].mean(axis=0))\n", ""),
    "retrieval_windows_from_segment_start": ("    last = q_prev[m - L:]", "    last = q_prev[:L]"),
    "retrieval_score_is_mean_over_summaries": ("scores = (sig @ k_pool.T).max(axis=0)", "scores = (sig @ k_pool.T).mean(axis=0)"),
    "retrieval_anchor_order_ascending": ("key=lambda r: (-scores[r], r))[:n_anchors]", "key=lambda r: (scores[r], r))[:n_anchors]"),
    "retrieval_window_not_clipped_left": ("for r in range(max(evicted, a_ - win_before), min(n, a_ + win_after + 1)):", "for r in range(a_ - win_before, min(n, a_ + win_after + 1)):"),
    "retrieval_window_one_short": ("min(n, a_ + win_after + 1)):", "min(n, a_ + win_after)):"),
    "retrieval_pads_with_latest": ("    r = evicted\n    while len(chosen) < want:\n        if r not in inside:\n            inside.add(r)\n            chosen.append(r)\n        r += 1", "    r = n - 1\n    while len(chosen) < want:\n        if r not in inside:\n            inside.add(r)\n            chosen.append(r)\n        r -= 1"),
    "retrieval_result_unsorted": ("res = np.array(sorted(chosen), dtype=np.int64)", "res = np.array(chosen, dtype=np.int64)"),
    "packed_segment_grid_runs_through_the_pack": ("            o, l = attend(q[None, lo:hi], k[None, lo:hi], v[None, lo:hi], **kw)\n            out[lo:hi], lse[:, lo:hi] = o[0], l[0]", "            o, l = attend(q[None, :hi], k[None, :hi], v[None, :hi], **kw)\n            out[lo:hi], lse[:, lo:hi] = o[0, lo:], l[0, :, lo:]"),
    "packed_lse_of_first_head_for_all": ("out[lo:hi], lse[:, lo:hi] = o[0], l[0]", "out[lo:hi], lse[:, lo:hi] = o[0], l[0, :1]"),
    "packed_backward_runs_through_the_pack": ("            gq, gk, gv = attend_backward(q[None, lo:hi], k[None, lo:hi], v[None, lo:hi], dout[None, lo:hi], **kw)\n            dq[lo:hi], dk[lo:hi], dv[lo:hi] = gq[0], gk[0], gv[0]", "            gq, gk, gv = attend_backward(q[None, :hi], k[None, :hi], v[None, :hi], dout[None, :hi], **kw)\n            dq[lo:hi], dk[lo:hi], dv[lo:hi] = gq[0, lo:], gk[0, lo:], gv[0, lo:]"),
    "bf16_rounding_truncates": ("np.rint(x / quantum)", "np.trunc(x / quantum)"),
    "bf16_rounding_ties_away_from_zero": ("np.rint(x / quantum)", "(np.sign(x) * np.floor(np.abs(x / quantum) + 0.5))"),
    "bf16_rounding_through_binary32": ("    x = np.asarray(x, dtype=np.float64)\n    _, e = np.frexp(x)", "    x = np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)\n    _, e = np.frexp(x)"),
    "bf16_grid_without_subnormal_floor": ("np.maximum(e - 8, -133)", "(e - 8)"),
    "bf16_grid_one_bit_too_fine": ("np.maximum(e - 8, -133)", "np.maximum(e - 9, -133)"),
    "bf16_overflow_saturates": ("np.copysign(np.inf, x), r)", "np.copysign(2.0 ** 127 * (2 - 2.0 ** -7), x), r)"),
    "tail_of_takes_head": ("return k_seg[m - t:], v_seg[m - t:]", "return k_seg[:t], v_seg[:t]"),
}


def _pin_calls():
    calls = []
    for name in sorted(dir(pins)):
        fn = getattr(pins, name)
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn, {}))
            continue
        combos = [{}]
        for m in marks:
            keys = [k.strip() for k in m.args[0].split(",")]
            new = []
            for vals in m.args[1]:
                vals = vals if isinstance(vals, (tuple, list)) and len(keys) > 1 else (vals,)
                for c in combos:
                    new.append({**c, **dict(zip(keys, vals))})
            combos = new
        calls.extend((name, fn, c) for c in combos)
    return calls


@pytest.mark.parametrize("mutant", sorted(MUTANTS))
def test_planted_mistake_is_caught(mutant, monkeypatch):
    old, new = MUTANTS[mutant]
    assert SRC.count(old) >= 1, "mutation site not found: oracle source changed"
    mod = types.ModuleType("oracle_mutant")
    exec(compile(SRC.replace(old, new), "oracle_mutant", "exec"), mod.__dict__)
    monkeypatch.setattr(pins, "orc", mod)
    failed = []
    for name, fn, kwargs in _pin_calls():
        try:
            fn(**kwargs)
        except (AssertionError, ValueError, IndexError, FloatingPointError, pytest.fail.Exception):
            failed.append(name)
    assert failed, f"no pin notices the planted mistake '{mutant}'"


def test_unmutated_oracle_passes_all_pins():
    for name, fn, kwargs in _pin_calls():
        fn(**kwargs)
