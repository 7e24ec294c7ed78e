"""Pins for the fp64 oracle: everything here checks oracle/ against something that is
NOT the oracle -- hand-computed fixtures, textbook loops written out below, closed forms
and invariants of Eq. 12 / Eq. 13 (Appendix C).  CPU only."""
import math

import numpy as np
import pytest

import workloads as W
from oracle import segattn_oracle as orc
from conftest import golden_path

POL = {"SEG": 0, "TAIL": 1, "PAST": 2, "TAIL|PAST": 3}


def _read(name):
    rows = []
    with open(golden_path(name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ---------------------------------------------------------------- independent references
def textbook_rows(q, k, v, scale, lo_of, hi_of):
    """Softmax attention of one head, key range [lo_of(p), hi_of(p)] per row, written as
    scalar Python loops (no matmul, no mask array): the textbook definition."""
    n, d = q.shape
    out = np.zeros((n, d))
    lse = np.zeros(n)
    for p in range(n):
        js = list(range(lo_of(p), hi_of(p) + 1))
        z = [scale * sum(q[p, c] * k[j, c] for c in range(d)) for j in js]
        zm = max(z)
        w = [math.exp(x - zm) for x in z]
        tot = sum(w)
        for c in range(d):
            out[p, c] = sum(wi * v[j, c] for wi, j in zip(w, js)) / tot
        lse[p] = zm + math.log(tot)
    return out, lse


def concat_formulation(q, k, v, S, T, policy, scale):
    """Literal Eq. 13: per segment build [prefix ; segment] by concatenation (prefix =
    carried tail for a local head, the whole earlier history for a long-range head,
    nothing otherwise), prefix fully visible, segment causal (Eq. 12's mask)."""
    n, d = q.shape
    out = np.zeros((n, d))
    lse = np.zeros(n)
    for s in range(0, n, S):
        m = min(S, n - s)
        if policy & 2:
            pk, pv = k[:s], v[:s]
        elif policy & 1:
            lo = max(0, s - T)
            pk, pv = k[lo:s], v[lo:s]
        else:
            pk, pv = k[:0], v[:0]
        kc = np.concatenate([pk, k[s:s + m]])
        vc = np.concatenate([pv, v[s:s + m]])
        P = pk.shape[0]
        for t in range(m):
            z = scale * (kc[:P + t + 1] @ q[s + t])
            w = np.exp(z - z.max())
            out[s + t] = (w / w.sum()) @ vc[:P + t + 1]
            lse[s + t] = z.max() + math.log(w.sum())
    return out, lse


# ---------------------------------------------------------------- hand-computed fixtures
def test_hand_case_constant_scores():
    v = np.arange(1.0, 7.0).reshape(1, 6, 1, 1)
    q = np.zeros((1, 6, 1, 1))
    k = _rand((1, 6, 1, 1), 0)          # irrelevant: q = 0
    for name, p, o_exp, cnt in _read("hand_case_constant_scores.txt"):
        o, l = orc.attend(q, k, v, seg_len=3, tail_len=1, kv_policy=[POL[name]])
        assert o[0, int(p), 0, 0] == pytest.approx(float(o_exp), abs=1e-14), (name, p)
        assert l[0, 0, int(p)] == pytest.approx(math.log(int(cnt)), abs=1e-14), (name, p)


def test_hand_case_log_keys():
    q = np.ones((1, 3, 1, 1))
    k = np.array([0.0, math.log(2), math.log(3)]).reshape(1, 3, 1, 1)
    v = np.array([1.0, 2.0, 3.0]).reshape(1, 3, 1, 1)
    o, l = orc.attend(q, k, v, seg_len=8, tail_len=0, kv_policy=[0], scale=1.0)
    for p, num, den, el in _read("hand_case_log_keys.txt"):
        assert o[0, int(p), 0, 0] == pytest.approx(int(num) / int(den), abs=1e-14)
        assert l[0, 0, int(p)] == pytest.approx(math.log(int(el)), abs=1e-14)


def test_default_scale_is_inverse_sqrt_d():
    # Eq. 12 divides by sqrt(d): with d=4, q=(1,1,1,1), k_j = c_j*(1,1,1,1): z_j = 4 c_j / 2.
    q = np.ones((1, 2, 1, 4))
    k = np.stack([np.zeros(4), np.full(4, math.log(3) / 2)]).reshape(1, 2, 1, 4)
    v = np.array([[0.0] * 4, [4.0] * 4]).reshape(1, 2, 1, 4)
    o, l = orc.attend(q, k, v, seg_len=2, tail_len=0, kv_policy=[0])
    assert l[0, 0, 1] == pytest.approx(math.log(1 + 3), abs=1e-14)      # exp(0)+exp(ln 3)
    assert o[0, 1, 0, 0] == pytest.approx(3.0, abs=1e-14)               # (0*1 + 4*3)/4


# ---------------------------------------------------------------- reductions to textbook loops
@pytest.mark.parametrize("policy", [0, 1, 2, 3])
def test_single_segment_is_plain_causal(policy):
    n, d = 13, 3
    q, k, v = _rand((n, d), 1), _rand((n, d), 2), _rand((n, d), 3)
    o, l = orc.attend(q[None, :, None], k[None, :, None], v[None, :, None],
                      seg_len=16, tail_len=5, kv_policy=[policy], scale=0.7)
    oe, le = textbook_rows(q, k, v, 0.7, lambda p: 0, lambda p: p)
    np.testing.assert_allclose(o[0, :, 0], oe, atol=1e-13)
    np.testing.assert_allclose(l[0, 0], le, atol=1e-13)


@pytest.mark.parametrize("policy", [2, 3])
def test_past_with_full_history_is_plain_causal(policy):
    n, d, S, T = 23, 2, 5, 2
    q, k, v = _rand((n, d), 4), _rand((n, d), 5), _rand((n, d), 6)
    o, l = orc.attend(q[None, :, None], k[None, :, None], v[None, :, None],
                      seg_len=S, tail_len=T, kv_policy=[policy])
    oe, le = textbook_rows(q, k, v, 1 / math.sqrt(d), lambda p: 0, lambda p: p)
    np.testing.assert_allclose(o[0, :, 0], oe, atol=1e-13)
    np.testing.assert_allclose(l[0, 0], le, atol=1e-13)


@pytest.mark.parametrize("T", [0, 1, 3, 7])
def test_tail_head_is_segment_banded(T):
    n, d, S = 26, 2, 7                     # ragged last segment (26 = 3*7 + 5)
    q, k, v = _rand((n, d), 7), _rand((n, d), 8), _rand((n, d), 9)
    o, l = orc.attend(q[None, :, None], k[None, :, None], v[None, :, None],
                      seg_len=S, tail_len=T, kv_policy=[1])
    lo = lambda p: max(0, (p // S) * S - T)
    oe, le = textbook_rows(q, k, v, 1 / math.sqrt(d), lo, lambda p: p)
    np.testing.assert_allclose(o[0, :, 0], oe, atol=1e-13)
    np.testing.assert_allclose(l[0, 0], le, atol=1e-13)


def test_seg_head_and_zero_tail_are_block_diagonal():
    n, d, S = 20, 3, 6
    q, k, v = _rand((n, d), 10), _rand((n, d), 11), _rand((n, d), 12)
    oe, le = textbook_rows(q, k, v, 1 / math.sqrt(d), lambda p: (p // S) * S, lambda p: p)
    for policy, T in ((0, 4), (1, 0)):
        o, l = orc.attend(q[None, :, None], k[None, :, None], v[None, :, None],
                          seg_len=S, tail_len=T, kv_policy=[policy])
        np.testing.assert_allclose(o[0, :, 0], oe, atol=1e-13)
        np.testing.assert_allclose(l[0, 0], le, atol=1e-13)


@pytest.mark.parametrize("policy", [0, 1, 2, 3])
@pytest.mark.parametrize("S,T,n", [(8, 0, 29), (8, 1, 32), (8, 8, 27), (5, 3, 64), (64, 16, 40)])
def test_mask_formulation_equals_concatenation_formulation(policy, S, T, n):
    d = 4
    q, k, v = _rand((n, d), 20 + n), _rand((n, d), 21 + n), _rand((n, d), 22 + n)
    o, l = orc.attend(q[None, :, None], k[None, :, None], v[None, :, None],
                      seg_len=S, tail_len=T, kv_policy=[policy])
    oe, le = concat_formulation(q, k, v, S, T, policy, 1 / math.sqrt(d))
    np.testing.assert_allclose(o[0, :, 0], oe, atol=1e-13)
    np.testing.assert_allclose(l[0, 0], le, atol=1e-13)


def test_gqa_head_map_and_batch_are_independent_problems():
    """Query head h reads KV head h // g; batches do not mix.  Each (b, h) must equal the
    single-head problem solved on its own."""
    B, n, Hq, Hkv, d, S, T = 2, 19, 6, 3, 4, 6, 2
    pol = [1, 3, 0]
    q, k, v = _rand((B, n, Hq, d), 30), _rand((B, n, Hkv, d), 31), _rand((B, n, Hkv, d), 32)
    o, l = orc.attend(q, k, v, seg_len=S, tail_len=T, kv_policy=pol)
    for b in range(B):
        for h in range(Hq):
            kv = h // 2
            oe, le = concat_formulation(q[b, :, h], k[b, :, kv], v[b, :, kv], S, T, pol[kv], 0.5)
            np.testing.assert_allclose(o[b, :, h], oe, atol=1e-13)
            np.testing.assert_allclose(l[b, h], le, atol=1e-13)


# ---------------------------------------------------------------- closed forms and invariants
def test_visible_pair_count_matches_cost_model_closed_form():
    for N, S, T, name, pairs in _read("visible_pairs_closed_form.txt"):
        N, S, T, pairs = int(N), int(S), int(T), int(pairs)
        n = N // S
        closed = n * S * (S + 1) // 2 + (n - 1) * S * T if name == "TAIL" else N * (N + 1) // 2
        assert closed == pairs
    # popcount of the oracle's mask against the same closed form (general m_i, ragged tail)
    for N, S, T in ((2048, 512, 128), (100, 16, 5), (77, 10, 10), (64, 8, 0)):
        starts = list(range(0, N, S))
        tail_pairs = sum((min(S, N - s) * (min(S, N - s) + 1)) // 2 + min(S, N - s) * min(T, s)
                         for s in starts)
        seg_pairs = sum((min(S, N - s) * (min(S, N - s) + 1)) // 2 for s in starts)
        assert orc.visible_pairs(N, S, T, 1) == tail_pairs
        assert orc.visible_pairs(N, S, T, 0) == seg_pairs
        assert orc.visible_pairs(N, S, T, 2) == N * (N + 1) // 2
        assert orc.visible_pairs(N, S, T, 3) == N * (N + 1) // 2
    assert orc.visible_pairs(2048, 512, 128, 1) == 721920


def test_effective_context_per_token_matches_cost_model():
    """Sec. 3.5: a local head's query sees at most S + M keys; a SEG head at most S."""
    N, S, T = 96, 16, 6
    assert max(orc.visible_mask(p, N, S, T, 1).sum() for p in range(N)) == S + T
    assert max(orc.visible_mask(p, N, S, T, 0).sum() for p in range(N)) == S
    assert max(orc.visible_mask(p, N, S, T, 2).sum() for p in range(N)) == N


def test_probabilities_sum_to_one_and_respect_mask():
    B, n, Hq, Hkv, d, S, T = 1, 37, 4, 4, 8, 8, 3
    q, k, v = _rand((B, n, Hq, d), 40), _rand((B, n, Hkv, d), 41), _rand((B, n, Hkv, d), 42)
    pol = [0, 1, 2, 3]
    o, l, pr = orc.attend(q, k, v, seg_len=S, tail_len=T, kv_policy=pol, return_probs=True)
    np.testing.assert_allclose(pr.sum(-1), 1.0, atol=1e-14)
    for h in range(4):
        for p in range(n):
            vis = orc.visible_mask(p, n, S, T, pol[h])
            assert np.all(pr[0, h, p][~vis] == 0.0)
            assert np.all(pr[0, h, p][vis] > 0.0)
            assert vis[p]                              # the diagonal is always visible


def test_zero_queries_give_mean_of_visible_values():
    n, Hkv, d, S, T = 41, 4, 5, 9, 4
    k, v = _rand((1, n, Hkv, d), 50), _rand((1, n, Hkv, d), 51)
    q = np.zeros((1, n, Hkv, d))
    pol = [0, 1, 2, 3]
    o, l = orc.attend(q, k, v, seg_len=S, tail_len=T, kv_policy=pol)
    for h in range(4):
        for p in range(n):
            vis = orc.visible_mask(p, n, S, T, pol[h])
            np.testing.assert_allclose(o[0, p, h], v[0, vis, h].mean(0), atol=1e-14)
            assert l[0, h, p] == pytest.approx(math.log(vis.sum()), abs=1e-14)


def test_shifting_all_keys_shifts_lse_only():
    """Adding one vector u to every key adds scale*q_p.u to every score of row p:
    O unchanged, LSE shifted by that constant."""
    n, d, S, T = 30, 6, 7, 3
    q, k, v = _rand((1, n, 2, d), 60), _rand((1, n, 2, d), 61), _rand((1, n, 2, d), 62)
    u = _rand((d,), 63)
    o1, l1 = orc.attend(q, k, v, seg_len=S, tail_len=T, kv_policy=[1, 3], scale=0.3)
    o2, l2 = orc.attend(q, k + u, v, seg_len=S, tail_len=T, kv_policy=[1, 3], scale=0.3)
    np.testing.assert_allclose(o1, o2, atol=1e-12)
    shift = 0.3 * np.einsum("bnhd,d->bhn", q, u)
    np.testing.assert_allclose(l2 - l1, shift, atol=1e-12)


def test_value_linearity_and_output_in_convex_hull():
    n, d, S, T = 25, 3, 6, 2
    q, k = _rand((1, n, 1, d), 70), _rand((1, n, 1, d), 71)
    v1, v2 = _rand((1, n, 1, d), 72), _rand((1, n, 1, d), 73)
    o1, _ = orc.attend(q, k, v1, seg_len=S, tail_len=T, kv_policy=[1])
    o2, _ = orc.attend(q, k, v2, seg_len=S, tail_len=T, kv_policy=[1])
    o12, _ = orc.attend(q, k, 2 * v1 - 3 * v2, seg_len=S, tail_len=T, kv_policy=[1])
    np.testing.assert_allclose(o12, 2 * o1 - 3 * o2, atol=1e-12)
    for p in range(n):
        vis = orc.visible_mask(p, n, S, T, 1)
        assert np.all(o1[0, p, 0] <= v1[0, vis, 0].max(0) + 1e-12)
        assert np.all(o1[0, p, 0] >= v1[0, vis, 0].min(0) - 1e-12)


def test_eviction_hides_oldest_past_rows_but_not_the_tail():
    n, d, S, T = 40, 3, 8, 3
    q, k, v = _rand((n, d), 80), _rand((n, d), 81), _rand((n, d), 82)
    ev = 13
    o, l = orc.attend(q[None, :, None], k[None, :, None], v[None, :, None],
                      seg_len=S, tail_len=T, kv_policy=[3], evicted=[ev])
    def lo(p):                     # [max(0,s-T), s) united with [ev, s): both end at s
        s = (p // S) * S
        return min(max(0, s - T), min(ev, s))
    oe, le = textbook_rows(q, k, v, 1 / math.sqrt(d), lo, lambda p: p)
    np.testing.assert_allclose(o[0, :, 0], oe, atol=1e-13)
    np.testing.assert_allclose(l[0, 0], le, atol=1e-13)


# ---------------------------------------------------------------- rows, decode, inputs
def test_row_subset_equals_rows_of_full_result():
    w = W.small(seq_len=70, seg_len=16, tail_len=5, n_q_heads=4, n_kv_heads=2, head_dim=8)
    q, k, v = W.prefill_inputs(w)
    o, l = orc.attend(q, k, v, seg_len=16, tail_len=5, kv_policy=w.kv_policy)
    rows = [0, 15, 16, 17, 69, 33]
    o2, l2 = orc.attend(q, k, v, seg_len=16, tail_len=5, kv_policy=w.kv_policy, rows=rows,
                        max_block_bytes=1500)
    np.testing.assert_array_equal(o2, o[:, rows])
    np.testing.assert_array_equal(l2, l[:, :, rows])


def test_decode_row_is_last_prefill_row():
    """Forward identity (Sec. 3.1): decoding token n-1 is row n-1 of prefilling n tokens."""
    n, Hq, Hkv, d, S, T = 45, 4, 2, 8, 16, 4
    q, k, v = _rand((1, n, Hq, d), 90), _rand((1, n, Hkv, d), 91), _rand((1, n, Hkv, d), 92)
    o, l = orc.attend(q, k, v, seg_len=S, tail_len=T, kv_policy=[1, 3])
    for m in (1, 16, 17, 32, 45):
        od, ld = orc.decode_attend(q[0, m - 1], k[0, :m], v[0, :m], seg_len=S, tail_len=T,
                                   kv_policy=[1, 3])
        np.testing.assert_allclose(od, o[0, m - 1], atol=1e-14)
        np.testing.assert_allclose(ld, l[0, :, m - 1], atol=1e-14)


def test_bf16_widening_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x3FC0, 0x0000, 0x4049, 0x3DCD], dtype=np.uint16)
    exp = [1.0, -1.0, 2.0, 1.5, 0.0, 3.140625, 0.10009765625]
    np.testing.assert_array_equal(orc.widen(bits), np.array(exp))


def _bf16_bits(x):
    """Bit patterns of float64 values that already are bfloat16 numbers (exact in binary32)."""
    return (np.asarray(x, dtype=np.float64).astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def test_round_bf16_matches_hand_worked_table():
    """Listed binary64 values against their hand-worked bfloat16 patterns: exact ties both ways,
    values a hair off a tie (which a detour over binary32 would misplace), both zeros,
    subnormals, the overflow threshold."""
    rows = _read("bf16_rounding_table.txt")
    assert len(rows) >= 25
    x = np.array([float.fromhex(r[0]) for r in rows])
    want = np.array([int(r[1], 16) for r in rows], dtype=np.uint16)
    got = orc.round_bf16(x)
    np.testing.assert_array_equal(_bf16_bits(got), want)
    np.testing.assert_array_equal(np.signbit(got), np.signbit(x))


def test_round_bf16_is_the_nearest_grid_point_and_idempotent():
    """Properties of round-to-nearest on any input: the result is a bfloat16 number (widening its
    own pattern gives it back), no other bfloat16 number is nearer (checked against the two
    neighbouring patterns), and rounding twice changes nothing."""
    rng = np.random.default_rng(17)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-30, 30, 4000),
                        rng.standard_normal(500) * 2.0 ** -130])
    r = orc.round_bf16(x)
    bits = _bf16_bits(r)
    np.testing.assert_array_equal(orc.widen(bits), r)
    np.testing.assert_array_equal(orc.round_bf16(r), r)
    mag = bits & np.uint16(0x7FFF)
    up = orc.widen(((mag + 1) | (bits & np.uint16(0x8000))).astype(np.uint16))          # next larger magnitude
    dn = orc.widen(((np.maximum(mag, 1) - 1) | (bits & np.uint16(0x8000))).astype(np.uint16))
    err = np.abs(r - x)
    assert np.all(err <= np.abs(up - x)) and np.all(err <= np.abs(dn - x))


def test_tail_of_is_last_rows():
    k = np.arange(10.0).reshape(5, 2)
    kt, vt = orc.tail_of(k, -k, 3)
    np.testing.assert_array_equal(kt, k[2:])
    kt, vt = orc.tail_of(k, -k, 8)
    np.testing.assert_array_equal(vt, -k)


def test_rejects_bad_arguments():
    q = np.zeros((1, 4, 2, 2))
    with pytest.raises(ValueError):
        orc.attend(q, q, q, seg_len=2, tail_len=3, kv_policy=[1, 1])       # T > S
    with pytest.raises(ValueError):
        orc.attend(q, q[:, :, :1], q, seg_len=2, tail_len=1, kv_policy=[1])  # V shape
    with pytest.raises(ValueError):
        orc.attend(q, q, q, seg_len=2, tail_len=1, kv_policy=[1, 1], rows=[4])


# ---------------------------------------------------------------- retrieved prefix
# Eq. 13, second case: a long-range head attends to [K_ret ; K_seg]; Appendix D "Output": the
# retrieved prefix is R gathered pool rows.  None of the references below touch the mask code.
def gathered_rows(q, k, v, S, ret_of_seg, scale):
    """Literal [gathered rows ; segment] with the textbook scalar loops: for the query at
    in-segment offset t, keys = the gathered rows in list order, then segment rows 0..t."""
    n, d = q.shape
    out = np.zeros((n, d))
    lse = np.zeros(n)
    for p in range(n):
        i, s = p // S, (p // S) * S
        js = [int(j) for j in ret_of_seg.get(i, ())] + list(range(s, p + 1))
        z = [scale * sum(q[p, c] * k[j, c] for c in range(d)) for j in js]
        zm = max(z)
        w = [math.exp(x - zm) for x in z]
        tot = sum(w)
        for c in range(d):
            out[p, c] = sum(wi * v[j, c] for wi, j in zip(w, js)) / tot
        lse[p] = zm + math.log(tot)
    return out, lse


def _random_retrieval(rng, n, S, R):
    """For every segment after the first, R (or fewer) distinct earlier positions in random order."""
    ret = {}
    for i in range(1, (n + S - 1) // S):
        s = i * S
        ret[i] = rng.permutation(s)[:min(R, s)]
    return ret


@pytest.mark.parametrize("S,R,n", [(8, 3, 29), (8, 8, 40), (5, 11, 33), (16, 1, 50)])
def test_retrieved_prefix_equals_literal_gather(S, R, n):
    d, B, Hkv, g = 3, 2, 2, 2
    rng = np.random.default_rng(300 + n)
    q = rng.standard_normal((B, n, Hkv * g, d))
    k, v = rng.standard_normal((B, n, Hkv, d)), rng.standard_normal((B, n, Hkv, d))
    per = {(b, h): _random_retrieval(rng, n, S, R) for b in range(B) for h in range(Hkv)}
    retrieved = {(b, h, i): idx for (b, h), r in per.items() for i, idx in r.items()}
    o, l = orc.attend(q, k, v, seg_len=S, tail_len=2, kv_policy=[2, 2], retrieved=retrieved)
    for b in range(B):
        for hq in range(Hkv * g):
            h = hq // g
            oe, le = gathered_rows(q[b, :, hq], k[b, :, h], v[b, :, h], S, per[(b, h)], 1 / math.sqrt(d))
            np.testing.assert_allclose(o[b, :, hq], oe, atol=1e-13)
            np.testing.assert_allclose(l[b, hq], le, atol=1e-13)


def test_retrieved_prefix_special_cases_reduce_to_the_other_policies():
    """Retrieving every earlier row is the full-history head, retrieving the last T rows of the
    previous segment is a local head, retrieving nothing is within-segment attention; a local
    head ignores the list."""
    n, d, S, T = 37, 4, 8, 3
    q, k, v = _rand((1, n, 1, d), 310), _rand((1, n, 1, d), 311), _rand((1, n, 1, d), 312)
    nseg = (n + S - 1) // S
    def run(policy, retrieved=None):
        return orc.attend(q, k, v, seg_len=S, tail_len=T, kv_policy=[policy], retrieved=retrieved)
    everything = {(0, 0, i): np.arange(i * S) for i in range(nseg)}
    window = {(0, 0, i): np.arange(max(0, i * S - T), i * S) for i in range(nseg)}
    for got, want in ((run(2, everything), run(2)), (run(2, window), run(1)), (run(2, {}), run(0)),
                      (run(1, everything), run(1))):
        np.testing.assert_allclose(got[0], want[0], atol=1e-13)
        np.testing.assert_allclose(got[1], want[1], atol=1e-13)
    lo = lambda p: (p // S) * S
    oe, le = textbook_rows(q[0, :, 0], k[0, :, 0], v[0, :, 0], 1 / math.sqrt(d), lo, lambda p: p)
    np.testing.assert_allclose(run(2, {})[0][0, :, 0], oe, atol=1e-13)


def test_retrieved_prefix_with_zero_queries_is_mean_of_gathered_and_segment_values():
    n, d, S = 20, 2, 6
    k, v = _rand((1, n, 1, d), 320), _rand((1, n, 1, d), 321)
    ret = {(0, 0, 1): [4, 0], (0, 0, 2): [11, 2, 7], (0, 0, 3): [17]}
    o, l = orc.attend(np.zeros((1, n, 1, d)), k, v, seg_len=S, tail_len=0, kv_policy=[2], retrieved=ret)
    for p in range(n):
        i, s = p // S, (p // S) * S
        js = list(ret.get((0, 0, i), [])) + list(range(s, p + 1))
        np.testing.assert_allclose(o[0, p, 0], v[0, js, 0].mean(0), atol=1e-14)
        assert abs(l[0, 0, p] - math.log(len(js))) < 1e-14


def test_retrieved_prefix_decode_row_and_bad_lists():
    n, d, S = 27, 4, 8
    q, k, v = _rand((1, n, 2, d), 330), _rand((1, n, 1, d), 331), _rand((1, n, 1, d), 332)
    ret = {(0, 0, i): np.random.default_rng(i).permutation(i * S)[:5] for i in range(1, 4)}
    o, l = orc.attend(q, k, v, seg_len=S, tail_len=0, kv_policy=[2], retrieved=ret)
    for m in (8, 9, 16, 27):
        od, ld = orc.decode_attend(q[0, m - 1], k[0, :m], v[0, :m], seg_len=S, tail_len=0, kv_policy=[2],
                                   retrieved={0: ret.get((0, 0, (m - 1) // S), ())})
        np.testing.assert_allclose(od, o[0, m - 1], atol=1e-14)
        np.testing.assert_allclose(ld, l[0, :, m - 1], atol=1e-14)
    with pytest.raises(ValueError):   # a row of the segment itself is not in the pool yet
        orc.attend(q, k, v, seg_len=S, tail_len=0, kv_policy=[2], retrieved={(0, 0, 1): [8]})
    with pytest.raises(ValueError):   # the same row twice would double its weight
        orc.attend(q, k, v, seg_len=S, tail_len=0, kv_policy=[2], retrieved={(0, 0, 1): [3, 3]})


# ---------------------------------------------------------------- backward
# Definition "K-truncated consistent objective" (Sec. 3.2) and the no-gradient lemma of
# Appendix B: the carried tail is differentiable, past rows are constants.  The reference is a
# scalar-loop forward in which the past rows come from separate, constant copies of K and V,
# differentiated numerically; it shares nothing with the oracle's formulas.
def split_forward_loss(q, k, v, k_const, v_const, gout, S, T, policy, scale):
    """sum(O * gout) for one head; a key seen through the tail or the own segment is read from
    (k, v), a key seen only through the PAST bit from (k_const, v_const)."""
    n, d = q.shape
    total = 0.0
    for p in range(n):
        s = (p // S) * S
        keys = []
        for j in range(0, p + 1):
            in_seg = j >= s
            in_tail = (policy & 1) and max(0, s - T) <= j < s
            in_past = (policy & 2) and j < s
            if in_seg or in_tail:
                keys.append((k[j], v[j]))
            elif in_past:
                keys.append((k_const[j], v_const[j]))
        z = np.array([scale * float(np.dot(q[p], kj)) for kj, _ in keys])
        w = np.exp(z - z.max())
        w /= w.sum()
        o = sum(wi * vj for wi, (_, vj) in zip(w, keys))
        total += float(np.dot(o, gout[p]))
    return total


def _numeric_grad(f, x, eps=1e-6):
    gr = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + eps
        fp = f()
        x[i] = old - eps
        fm = f()
        x[i] = old
        gr[i] = (fp - fm) / (2 * eps)
    return gr


@pytest.mark.parametrize("policy", [0, 1, 2, 3])
@pytest.mark.parametrize("S,T,n", [(4, 2, 11), (5, 5, 12), (16, 3, 9)])
def test_backward_equals_numerical_gradient_with_past_rows_constant(policy, S, T, n):
    d = 3
    rng = np.random.default_rng(400 + 10 * policy + n)
    q, k, v, go = (rng.standard_normal((n, d)) for _ in range(4))
    kc, vc = k.copy(), v.copy()
    scale = 0.7
    f = lambda: split_forward_loss(q, k, v, kc, vc, go, S, T, policy, scale)
    want = [_numeric_grad(f, x) for x in (q, k, v)]
    got = orc.attend_backward(q[None, :, None], k[None, :, None], v[None, :, None], go[None, :, None],
                              seg_len=S, tail_len=T, kv_policy=[policy], scale=scale)
    for g_, w_ in zip(got, want):
        np.testing.assert_allclose(g_[0, :, 0], w_, atol=2e-8)


def test_backward_sums_the_query_heads_of_a_group_and_keeps_sequences_apart():
    n, d, S, T, B, Hkv, g = 10, 2, 4, 2, 2, 2, 2
    rng = np.random.default_rng(410)
    q, go = rng.standard_normal((B, n, Hkv * g, d)), rng.standard_normal((B, n, Hkv * g, d))
    k, v = rng.standard_normal((B, n, Hkv, d)), rng.standard_normal((B, n, Hkv, d))
    pol = [1, 3]
    dq, dk, dv = orc.attend_backward(q, k, v, go, seg_len=S, tail_len=T, kv_policy=pol)
    for b in range(B):
        for h in range(Hkv):
            dk_sum, dv_sum = np.zeros((n, d)), np.zeros((n, d))
            for hq in range(h * g, (h + 1) * g):
                one = orc.attend_backward(q[b:b + 1, :, hq:hq + 1], k[b:b + 1, :, h:h + 1], v[b:b + 1, :, h:h + 1],
                                          go[b:b + 1, :, hq:hq + 1], seg_len=S, tail_len=T, kv_policy=[pol[h]])
                np.testing.assert_allclose(dq[b, :, hq], one[0][0, :, 0], atol=1e-14)
                dk_sum += one[1][0, :, 0]
                dv_sum += one[2][0, :, 0]
            np.testing.assert_allclose(dk[b, :, h], dk_sum, atol=1e-13)
            np.testing.assert_allclose(dv[b, :, h], dv_sum, atol=1e-13)


def test_backward_closed_forms():
    """(i) Uniform attention (Q = 0): dV_j = sum over the queries that see j of dout_i / |vis(i)|,
    and sum_j dV_j = sum_i dout_i when every visible pair is differentiable.  (ii) dout = 0 gives
    zero gradients.  (iii) Row blocking does not change the result.  (iv) Forward-only rows."""
    n, d, S, T = 13, 3, 5, 2
    rng = np.random.default_rng(420)
    k, v, go = (rng.standard_normal((1, n, 1, d)) for _ in range(3))
    q0 = np.zeros((1, n, 1, d))
    dq, dk, dv = orc.attend_backward(q0, k, v, go, seg_len=S, tail_len=T, kv_policy=[1])
    want = np.zeros((n, d))
    for p in range(n):
        vis = orc.visible_mask(p, n, S, T, 1)
        want[vis] += go[0, p, 0] / vis.sum()
    np.testing.assert_allclose(dv[0, :, 0], want, atol=1e-14)
    np.testing.assert_allclose(dv.sum(axis=1), go.sum(axis=1), atol=1e-13)
    q = rng.standard_normal((1, n, 1, d))
    for gr in orc.attend_backward(q, k, v, np.zeros_like(go), seg_len=S, tail_len=T, kv_policy=[3]):
        assert not gr.any()
    a = orc.attend_backward(q, k, v, go, seg_len=S, tail_len=T, kv_policy=[3])
    b = orc.attend_backward(q, k, v, go, seg_len=S, tail_len=T, kv_policy=[3], max_block_bytes=8 * n * 4)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, atol=1e-14)
    # a PAST-only head: later segments read the rows of segment 0 forward-only, so those rows get
    # exactly the gradient of the 5-token problem made of segment 0 alone
    _, dk2, dv2 = orc.attend_backward(q, k, v, go, seg_len=S, tail_len=T, kv_policy=[2])
    alone = orc.attend_backward(q[:, :S], k[:, :S], v[:, :S], go[:, :S], seg_len=S, tail_len=T, kv_policy=[0])
    np.testing.assert_allclose(dk2[0, :S, 0], alone[1][0, :, 0], atol=1e-14)
    np.testing.assert_allclose(dv2[0, :S, 0], alone[2][0, :, 0], atol=1e-14)


# ---------------------------------------------------------------- RoPE re-indexing (Appendix E)
def test_rope_hand_values_and_textbook_properties():
    # D = 2: one pair, frequency theta^0 = 1: rotation of (x0, x1) by `position` radians
    x = np.array([[[[1.0, 0.0]]], [[[0.0, 2.0]]], [[[3.0, 4.0]]]]).reshape(3, 1, 2)
    y = orc.rope_rotate(x, [0, 1, 2], theta=10000.0)
    np.testing.assert_allclose(y[0, 0], [1.0, 0.0], atol=1e-15)                       # position 0: identity
    np.testing.assert_allclose(y[1, 0], [-2 * math.sin(1), 2 * math.cos(1)], atol=1e-15)
    np.testing.assert_allclose(y[2, 0], [3 * math.cos(2) - 4 * math.sin(2), 3 * math.sin(2) + 4 * math.cos(2)], atol=1e-15)
    # D = 4, theta = 100: pairs (0,2) at frequency 1 and (1,3) at frequency 100^(-1/2) = 0.1
    x4 = np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 1, 4)
    y4 = orc.rope_rotate(x4, [5], theta=100.0)[0, 0]
    want = [math.cos(5) - 3 * math.sin(5), 2 * math.cos(0.5) - 4 * math.sin(0.5),
            math.sin(5) + 3 * math.cos(5), 2 * math.sin(0.5) + 4 * math.cos(0.5)]
    np.testing.assert_allclose(y4, want, atol=1e-14)
    # norm preserved; inner products depend on the position difference only
    rng = np.random.default_rng(500)
    a, b = rng.standard_normal((1, 1, 16)), rng.standard_normal((1, 1, 16))
    np.testing.assert_allclose(np.linalg.norm(orc.rope_rotate(a, [12345])), np.linalg.norm(a), rtol=1e-13)
    d1 = float(orc.rope_rotate(a, [70])[0, 0] @ orc.rope_rotate(b, [50])[0, 0])
    d2 = float(orc.rope_rotate(a, [1020])[0, 0] @ orc.rope_rotate(b, [1000])[0, 0])
    d3 = float(orc.rope_rotate(a, [71])[0, 0] @ orc.rope_rotate(b, [50])[0, 0])
    assert abs(d1 - d2) < 1e-12 and abs(d1 - d3) > 1e-3


@pytest.mark.parametrize("policy", [0, 1, 2, 3])
def test_reindexed_positions_equal_absolute_positions_for_contiguous_prefixes(policy):
    """A prefix that is a contiguous run of tokens ending at the segment start keeps every
    query-key distance under re-indexing, so Appendix E's positions give exactly standard RoPE
    with absolute positions followed by the unrotated-path attention."""
    n, d, S, T = 29, 8, 8, 3
    rng = np.random.default_rng(510 + policy)
    q, k, v = rng.standard_normal((1, n, 2, d)), rng.standard_normal((1, n, 1, d)), rng.standard_normal((1, n, 1, d))
    o1, l1 = orc.attend_reindexed(q, k, v, seg_len=S, tail_len=T, kv_policy=[policy], theta=50.0)
    qa, ka = orc.rope_rotate(q, np.arange(n), 50.0), orc.rope_rotate(k, np.arange(n), 50.0)
    o2, l2 = orc.attend(qa, ka, v, seg_len=S, tail_len=T, kv_policy=[policy])
    np.testing.assert_allclose(o1, o2, atol=1e-12)
    np.testing.assert_allclose(l1, l2, atol=1e-12)


def test_reindexed_retrieved_prefix_is_the_literal_concatenation():
    """Retrieved rows take positions 0..R-1 in list order and the segment R..R+m-1 (Appendix E,
    P = R), checked against scalar loops; unlike a contiguous prefix this is *not* what absolute
    positions would give."""
    n, d, S, theta = 20, 4, 6, 30.0
    rng = np.random.default_rng(520)
    q, k, v = rng.standard_normal((n, d)), rng.standard_normal((n, d)), rng.standard_normal((n, d))
    ret = {(0, 0, 1): [4, 0, 2], (0, 0, 2): [11, 3], (0, 0, 3): [17, 1, 9, 5]}
    o, l = orc.attend_reindexed(q[None, :, None], k[None, :, None], v[None, :, None], seg_len=S, tail_len=0,
                                kv_policy=[2], theta=theta, retrieved=ret)
    def rot(x, pos):
        h = d // 2
        y = np.zeros(d)
        for i in range(h):
            a = pos * theta ** (-2.0 * i / d)
            y[i] = x[i] * math.cos(a) - x[i + h] * math.sin(a)
            y[i + h] = x[i] * math.sin(a) + x[i + h] * math.cos(a)
        return y
    for p in range(n):
        i, s = p // S, (p // S) * S
        pref = list(ret.get((0, 0, i), []))
        P = len(pref)
        keys = [rot(k[j], u) for u, j in enumerate(pref)] + [rot(k[j], P + j - s) for j in range(s, p + 1)]
        vals = [v[j] for j in pref] + [v[j] for j in range(s, p + 1)]
        qq = rot(q[p], P + p - s)
        z = np.array([float(qq @ kk) / math.sqrt(d) for kk in keys])
        w = np.exp(z - z.max())
        np.testing.assert_allclose(o[0, p, 0], (w / w.sum()) @ np.array(vals), atol=1e-13)
        assert abs(l[0, 0, p] - (z.max() + math.log(w.sum()))) < 1e-13
    qa, ka = orc.rope_rotate(q[None, :, None], np.arange(n), theta), orc.rope_rotate(k[None, :, None], np.arange(n), theta)
    o_abs, _ = orc.attend(qa, ka, v[None, :, None], seg_len=S, tail_len=0, kv_policy=[2], retrieved=ret)
    assert np.abs(o_abs - o).max() > 1e-3


# ---------------------------------------------------------------- retrieval operator (Appendix D)
# The paper states the steps but none of the sizes, so these pins tie the oracle's reading to
# the literal description of the steps, not to printed values ("parity unpinned" w.r.t. the paper).
RET = dict(n_queries=6, pool_window=2, tail_avg=2, n_anchors=2, win_before=1, win_after=1)


def test_retrieval_summaries_by_hand():
    q = np.arange(1.0, 9.0).reshape(8, 1, 1)                 # rows 1..8, one head, D = 1
    s = orc.retrieval_summaries(q, n_queries=6, pool_window=4, tail_avg=3)
    # last 6 rows: 3..8 -> windows (3,4,5,6) and (7,8); tail mean of (6,7,8)
    np.testing.assert_allclose(s[:, 0, 0], [4.5, 7.5, 7.0])
    s = orc.retrieval_summaries(q[:3], n_queries=6, pool_window=2, tail_avg=5)   # fewer rows than L_q
    np.testing.assert_allclose(s[:, 0, 0], [1.5, 3.0, 2.0])


def literal_appendix_d(q_prev, k_pool, R, k_top, p):
    """Appendix D step by step: per summary take the top-k rows, de-duplicate the union, keep the
    n_anchors highest-scoring ones as anchors, expand, de-duplicate / sort, pad with the earliest
    rows.  Scores and window rules as in the oracle's docstring; plain Python sets and sorts."""
    summ = orc.round_bf16(orc.retrieval_summaries(q_prev, n_queries=p["n_queries"], pool_window=p["pool_window"],
                                                  tail_avg=p["tail_avg"]))
    sig = summ.reshape(-1, summ.shape[-1])
    n = k_pool.shape[0]
    per = [[float(np.dot(sg, k_pool[r])) for r in range(n)] for sg in sig]
    union = set()
    for sc in per:
        union |= set(sorted(range(n), key=lambda r: (-sc[r], r))[:k_top])
    best = {r: max(sc[r] for sc in per) for r in union}
    anchors = sorted(union, key=lambda r: (-best[r], r))[:p["n_anchors"]]
    picked = []
    for a_ in anchors:
        for r in range(max(0, a_ - p["win_before"]), min(n, a_ + p["win_after"] + 1)):
            if r not in picked and len(picked) < min(R, n):
                picked.append(r)
    r = 0
    while len(picked) < min(R, n):
        if r not in picked:
            picked.append(r)
        r += 1
    return sorted(picked)


@pytest.mark.parametrize("seed,n,R,k_top", [(1, 40, 8, 2), (2, 64, 10, 5), (3, 17, 12, 3), (4, 9, 20, 2), (5, 50, 3, 4)])
def test_retrieve_indices_equals_literal_steps(seed, n, R, k_top):
    rng = np.random.default_rng(600 + seed)
    q_prev = orc.round_bf16(rng.standard_normal((11, 2, 8)))
    k_pool = orc.round_bf16(rng.standard_normal((n, 8)))
    got = orc.retrieve_indices(q_prev, k_pool, R=R, **RET)
    assert list(got) == literal_appendix_d(q_prev, k_pool, R, k_top, RET)
    assert len(got) == min(R, n) and len(set(got)) == len(got) and list(got) == sorted(got)


def test_bf16_summaries_change_the_result_only_in_near_ties():
    """The summaries' precision is a reading (Appendix D states none).  Rounding a summary to bf16
    moves each of its components by at most 2^-8 relative (half a spacing of 2^-7), hence a row's score by at most
    eps_r = 2^-8 max_summary sum_d |s_d k_rd|.  Whenever the n_anchors + 1 best float64 scores are
    further apart than twice the largest eps, both readings must pick the same anchors in the same
    order and so return the same list; only closer calls may differ."""
    separated = differing = 0
    for seed in range(60):
        rng = np.random.default_rng(7000 + seed)
        n = int(rng.integers(12, 80))
        q_prev = orc.round_bf16(rng.standard_normal((9, 2, 8)))
        k_pool = orc.round_bf16(rng.standard_normal((n, 8)))
        R = int(rng.integers(2, 10))
        a, sa_ = orc.retrieve_indices(q_prev, k_pool, R=R, return_scores=True, **RET)
        b, sb = orc.retrieve_indices(q_prev, k_pool, R=R, return_scores=True, summaries_bf16=False, **RET)
        summ = orc.retrieval_summaries(q_prev, n_queries=RET["n_queries"], pool_window=RET["pool_window"],
                                       tail_avg=RET["tail_avg"]).reshape(-1, 8)
        eps = 2.0 ** -8 * (np.abs(summ) @ np.abs(k_pool).T).max(axis=0)
        assert np.all(np.abs(sa_ - sb) <= eps + 1e-15)
        top = np.sort(sb)[::-1][:RET["n_anchors"] + 1]
        if np.all(top[:-1] - top[1:] > 2 * eps.max()):
            separated += 1
            assert list(a) == list(b), seed
        elif list(a) != list(b):
            differing += 1
    assert separated >= 30          # the claim is not vacuous on this data


def test_retrieve_indices_planted_rows_and_fallback():
    """Keys equal to a multiple of the (single) summary direction win; windows of 3 rows around
    two anchors give 6 rows, the earliest rows pad to R = 9; evicted rows are never returned."""
    d, n = 4, 30
    q_prev = np.tile(np.array([1.0, 0.0, 0.0, 0.0]), (6, 1, 1))            # every summary = e0
    k_pool = np.zeros((n, d))
    k_pool[:, 1] = 1.0
    k_pool[20, 0], k_pool[11, 0] = 5.0, 3.0
    got = orc.retrieve_indices(q_prev, k_pool, R=9, **RET)
    assert list(got) == [0, 1, 2, 10, 11, 12, 19, 20, 21]
    got = orc.retrieve_indices(q_prev, k_pool, R=4, **RET)                  # best anchor first, then truncation
    assert list(got) == [10, 19, 20, 21]
    got = orc.retrieve_indices(q_prev, k_pool, R=9, evicted=11, **RET)     # row 11 itself is the first kept row
    assert list(got) == [11, 12, 13, 14, 15, 16, 19, 20, 21]
    k_pool[29, 0] = 9.0                                                     # window clipped at the pool end
    got = orc.retrieve_indices(q_prev, k_pool, R=5, **RET)
    assert list(got) == [19, 20, 21, 28, 29]


def test_packed_batch_keeps_sequences_apart_and_restarts_the_segment_grid():
    """A packed ragged batch is a set of independent samples: equal lengths reproduce the dense
    batch; a sequence's result does not change when its neighbours do; and the segment grid starts
    again at each sequence's first row (a one-segment sequence is plain causal attention whatever
    precedes it in the pack)."""
    rng = np.random.default_rng(77)
    Hq, Hkv, D, S, T = 4, 2, 8, 5, 2
    kw = dict(seg_len=S, tail_len=T, kv_policy=[1, 3])
    n = 12
    q, k, v = (rng.standard_normal((3, n, h, D)) for h in (Hq, Hkv, Hkv))
    o_d, l_d = orc.attend(q, k, v, **kw)
    cu = np.arange(4) * n
    o_p, l_p = orc.attend_packed(q.reshape(3 * n, Hq, D), k.reshape(3 * n, Hkv, D), v.reshape(3 * n, Hkv, D), cu, **kw)
    np.testing.assert_array_equal(o_p.reshape(3, n, Hq, D), o_d)
    np.testing.assert_array_equal(l_p.reshape(Hq, 3, n).transpose(1, 0, 2), l_d)

    lens = [7, 0, 4, 11]
    cu = np.concatenate([[0], np.cumsum(lens)])
    tot = int(cu[-1])
    q, k, v = (rng.standard_normal((tot, h, D)) for h in (Hq, Hkv, Hkv))
    o1, l1 = orc.attend_packed(q, k, v, cu, **kw)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    for x in (q2, k2, v2):
        x[:7] += 1.0            # disturb sequence 0 only
    o2, l2 = orc.attend_packed(q2, k2, v2, cu, **kw)
    np.testing.assert_array_equal(o1[7:], o2[7:])
    np.testing.assert_array_equal(l1[:, 7:], l2[:, 7:])
    assert np.abs(o1[:7] - o2[:7]).max() > 1e-3
    # sequence 2 (4 rows < S) sits at packed rows 7..10, across a multiple of S of the pack: it
    # must be plain causal softmax attention over its own rows
    lo = 7
    for t in range(4):
        for h in range(Hq):
            sc = (k[lo:lo + t + 1, h // 2] @ q[lo + t, h]) / math.sqrt(D)
            pr = np.exp(sc - sc.max())
            pr /= pr.sum()
            np.testing.assert_allclose(o1[lo + t, h], pr @ v[lo:lo + t + 1, h // 2], rtol=0, atol=1e-12)


def test_packed_backward_is_the_gradient_of_the_packed_forward():
    """attend_backward_packed against central differences of L = sum(attend_packed(...) * dO):
    the gradient of a packed batch, including that nothing leaks across sequence boundaries
    (TAIL | SEG policies only: no forward-only rows, so the full gradient is the paper's)."""
    rng = np.random.default_rng(78)
    Hq, Hkv, D, S, T = 2, 1, 4, 3, 2
    kw = dict(seg_len=S, tail_len=T, kv_policy=[1])
    lens = [5, 0, 2, 7]
    cu = np.concatenate([[0], np.cumsum(lens)])
    tot = int(cu[-1])
    q, k, v, g = (rng.standard_normal((tot, h, D)) for h in (Hq, Hkv, Hkv, Hq))

    def loss(q_, k_, v_):
        o, _ = orc.attend_packed(q_, k_, v_, cu, **kw)
        return float((o * g).sum())

    dq, dk, dv = orc.attend_backward_packed(q, k, v, g, cu, **kw)
    eps = 1e-6
    for name, x, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for idx in [(0, 0, 1), (4, 0, 3), (5, 0, 0), (6, 0, 2), (7, 0, 1), (13, 0, 0)]:
            if idx[1] >= x.shape[1]:
                continue
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])
