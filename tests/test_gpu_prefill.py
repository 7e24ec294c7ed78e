"""GPU parity: seg_attn_fwd_seq / seg_attn_fwd + seg_kv_commit against the fp64 oracle,
element by element on the same seeded inputs, through the C ABI."""
import numpy as np
import pytest

import workloads as W
from oracle import segattn_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _oracle(w, q, k, v, rows=None, scale=None):
    return orc.attend(q, k, v, seg_len=w.seg_len, tail_len=w.tail_len, kv_policy=w.kv_policy,
                      rows=rows, scale=scale)


SMALL = [
    # name, kwargs: sizes span several 64-key tiles, ragged tails, every policy, GQA 1/2/4/8
    dict(seq_len=200, seg_len=64, tail_len=16, n_q_heads=4, n_kv_heads=4, head_dim=64),
    dict(seq_len=333, seg_len=100, tail_len=37, n_q_heads=8, n_kv_heads=4, head_dim=128),
    dict(seq_len=700, seg_len=256, tail_len=256, n_q_heads=16, n_kv_heads=4, head_dim=128),
    dict(seq_len=513, seg_len=512, tail_len=0, n_q_heads=8, n_kv_heads=1, head_dim=64),
    dict(seq_len=96, seg_len=128, tail_len=32, n_q_heads=3, n_kv_heads=1, head_dim=128),
    dict(seq_len=1, seg_len=8, tail_len=8, n_q_heads=4, n_kv_heads=4, head_dim=64),
    dict(seq_len=450, seg_len=70, tail_len=70, n_q_heads=24, n_kv_heads=4, head_dim=128, batch=2),
]


@pytest.fixture(params=["auto", "4", "8"])
def waves(request, monkeypatch):
    """Workgroup shape of the head_dim-128 MFMA kernel: the library's own choice, or forced."""
    import gpu_util as G
    monkeypatch.setitem(G.TUNING, "prefill_waves", 0 if request.param == "auto" else int(request.param))
    return request.param


@pytest.mark.parametrize("fp32_check", [True, False])
@pytest.mark.parametrize("case", range(len(SMALL)))
def test_fwd_seq_small(case, fp32_check, waves):
    import gpu_util as G
    if waves != "auto" and (fp32_check or SMALL[case]["head_dim"] != 128):
        pytest.skip("the wave count only exists in the head_dim-128 MFMA kernel")
    w = W.small(f"small{case}", index=100 + case, **SMALL[case])
    q, k, v = W.prefill_inputs(w)
    o_ref, l_ref = _oracle(w, q, k, v)
    o, l = G.fwd_seq(w, q, k, v, fp32_check=fp32_check)
    G.assert_parity(o, l, o_ref, l_ref, fp32_check=fp32_check, what=f"small{case}")


@pytest.mark.parametrize("item_queues", [1, 2])
@pytest.mark.parametrize("seq_len,seg_len,tail_len", [(1400, 640, 200), (1100, 1100, 0), (2000, 512, 512)])
def test_fwd_seq_items_of_many_steps(seq_len, seg_len, tail_len, item_queues, monkeypatch):
    """Items of 2 to 60 key steps, every row against the oracle: the eight-wave kernel runs its
    unmasked steps in blocks of eight at fixed ring positions, so an item's length decides how many
    blocks it has (0 to 7), how many steps are left for the pairwise loop behind them, and where the
    prefix ends inside a block (tail_len 200: a ragged prefix; 0: none; 512: whole steps)."""
    import gpu_util as G
    monkeypatch.setitem(G.TUNING, "prefill_waves", 8)
    monkeypatch.setitem(G.TUNING, "item_queues", item_queues)
    w = W.small("long_items", index=150, seq_len=seq_len, seg_len=seg_len, tail_len=tail_len, n_q_heads=8,
                n_kv_heads=2, head_dim=128, kv_policy=[3, 1])
    q, k, v = W.prefill_inputs(w)
    o_ref, l_ref = _oracle(w, q, k, v)
    o, l = G.fwd_seq(w, q, k, v, fp32_check=False)
    G.assert_parity(o, l, o_ref, l_ref, fp32_check=False, what="long items")


@pytest.mark.parametrize("fp32_check", [True, False])
def test_fwd_seq_c1_full(fp32_check):
    import gpu_util as G
    w = W.C1
    q, k, v = W.prefill_inputs(w)
    o_ref, l_ref = _oracle(w, q, k, v)
    o, l = G.fwd_seq(w, q, k, v, fp32_check=fp32_check)
    G.assert_parity(o, l, o_ref, l_ref, fp32_check=fp32_check, what="C1")


@pytest.mark.parametrize("fp32_check", [True, False])
def test_packed_ragged_batch_matches_per_sequence_oracle(fp32_check, waves):
    """seg_attn_fwd_varlen: sequences of different lengths packed without padding, each with its own
    segment grid; the oracle is run sequence by sequence."""
    import gpu_util as G
    if waves != "auto" and fp32_check:
        pytest.skip("the wave count only exists in the head_dim-128 MFMA kernel")
    lens = [300, 1, 0, 513, 128, 77]
    S, T = 128, 32
    w = W.small("ragged", index=140, seq_len=sum(lens), seg_len=S, tail_len=T, n_q_heads=8, n_kv_heads=4,
                head_dim=128, kv_policy=[1, 3, 0, 2])
    q, k, v = W.prefill_inputs(w)                       # [1, total, H, D]: one stream, cut into sequences
    total = sum(lens)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cfg = G.config_of(w, fp32_check=fp32_check, out_fp32=True, batch=len(lens))
    qd, kd, vd = G.dev_bf16(q[0]), G.dev_bf16(k[0]), G.dev_bf16(v[0])
    out = torch.full((total, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((8, total), float("nan"), dtype=torch.float32, device="cuda")
    G.sa.seg_attn_fwd_varlen(cfg, qd, kd, vd, torch.from_numpy(cu).cuda(), total, max(lens), out, lse,
                           torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    o_gpu, l_gpu = G.to_f64(out), G.to_f64(lse)
    o_ref, l_ref = orc.attend_packed(q[0], k[0], v[0], cu, seg_len=S, tail_len=T, kv_policy=w.kv_policy)
    for b, n in enumerate(lens):
        lo, hi = int(cu[b]), int(cu[b + 1])
        if n:
            G.assert_parity(o_gpu[lo:hi], l_gpu[:, lo:hi], o_ref[lo:hi], l_ref[:, lo:hi], fp32_check=fp32_check,
                            what=f"ragged sequence {b} (n={n})")


def test_packed_batch_of_one_equals_the_dense_call_and_max_seqlen_only_sizes_the_launch():
    """A pack that holds a single sequence is the dense problem: same kernel, same order of
    operations, so the results are bit-identical; max_seqlen only sizes the launch, so a value
    above the longest sequence (up to the total) changes nothing."""
    import gpu_util as G
    w = W.small("one", index=141, seq_len=700, seg_len=256, tail_len=64, n_q_heads=8, n_kv_heads=2, head_dim=128)
    q, k, v = W.prefill_inputs(w)
    cfg = G.config_of(w, out_fp32=True, batch=1)
    qd, kd, vd = G.dev_bf16(q), G.dev_bf16(k), G.dev_bf16(v)
    st = torch.cuda.current_stream().cuda_stream
    o1 = torch.empty((1, 700, 8, 128), dtype=torch.float32, device="cuda")
    l1 = torch.empty((1, 8, 700), dtype=torch.float32, device="cuda")
    G.sa.seg_attn_fwd_seq(cfg, qd, kd, vd, 700, o1, l1, st)
    cu = torch.tensor([0, 700], dtype=torch.int32, device="cuda")
    o2 = torch.full((700, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    l2 = torch.full((8, 700), float("nan"), dtype=torch.float32, device="cuda")
    G.sa.seg_attn_fwd_varlen(cfg, qd[0], kd[0], vd[0], cu, 700, 700, o2, l2, st)
    torch.cuda.synchronize()
    assert torch.equal(o1[0], o2) and torch.equal(l1[0], l2)
    # two sequences: the launch sized by the longest (400) or by more than that (700)
    cfg2 = G.config_of(w, out_fp32=True, batch=2)
    cu2 = torch.tensor([0, 300, 700], dtype=torch.int32, device="cuda")
    res = []
    for max_len in (400, 700):
        o3 = torch.full((700, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
        l3 = torch.full((8, 700), float("nan"), dtype=torch.float32, device="cuda")
        G.sa.seg_attn_fwd_varlen(cfg2, qd[0], kd[0], vd[0], cu2, 700, max_len, o3, l3, st)
        torch.cuda.synchronize()
        res.append((o3, l3))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])
    assert bool(torch.isfinite(res[0][0]).all())
    with pytest.raises(G.sa.SegattnError):
        G.sa.seg_attn_fwd_varlen(cfg, qd[0], kd[0], vd[0], cu, 700, 701, o2, l2, st)   # max_seqlen > total


def test_stateless_forward_replays_from_a_captured_graph():
    """seg_attn_fwd_seq enqueues kernels only: captured once (after a warm-up call, which sets the
    kernel's shared-memory attribute), every replay on new inputs must equal the eager result,
    with eager launches and synchronisations between the replays."""
    import gpu_util as G
    w = W.small("graph", index=142, seq_len=900, seg_len=256, tail_len=64, n_q_heads=8, n_kv_heads=2, head_dim=128,
                kv_policy=[3, 1])
    cfg = G.config_of(w, out_fp32=True, batch=1)
    q, k, v = W.prefill_inputs(w)
    qd, kd, vd = G.dev_bf16(q), G.dev_bf16(k), G.dev_bf16(v)
    out = torch.empty((1, 900, 8, 128), dtype=torch.float32, device="cuda")
    lse = torch.empty((1, 8, 900), dtype=torch.float32, device="cuda")
    out_e, lse_e = torch.empty_like(out), torch.empty_like(lse)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        G.sa.seg_attn_fwd_seq(cfg, qd, kd, vd, 900, out, lse, side.cuda_stream)   # warm-up outside the capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        G.sa.seg_attn_fwd_seq(cfg, qd, kd, vd, 900, out, lse, torch.cuda.current_stream().cuda_stream)
    gen = torch.Generator(device="cuda").manual_seed(7)
    for _ in range(4):
        for t in (qd, kd, vd):   # new inputs in the captured buffers
            t.copy_(torch.randn(t.shape, device="cuda", generator=gen).to(torch.bfloat16))
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        G.sa.seg_attn_fwd_seq(cfg, qd, kd, vd, 900, out_e, lse_e, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert torch.equal(out, out_e) and torch.equal(lse, lse_e)
    bits = [t.view(torch.int16).cpu().numpy().view(np.uint16) for t in (qd, kd, vd)]   # the last inputs
    o_ref, l_ref = _oracle(w, *bits)
    G.assert_parity(G.to_f64(out), G.to_f64(lse), o_ref, l_ref, fp32_check=False, what="graph replay")


# ---- work items taken from queues (the form a launch with more items than fit the chip uses;
# ---- segattn_config.item_queues = 3 forces it for small inputs, = 1 switches it off)
@pytest.mark.parametrize("case", range(len(SMALL)))
def test_fwd_seq_small_with_item_queues(case, monkeypatch):
    import gpu_util as G
    monkeypatch.setitem(G.TUNING, "item_queues", G.QUEUES_ON_SMALL_GRID)
    w = W.small(f"small{case}", index=100 + case, **SMALL[case])
    q, k, v = W.prefill_inputs(w)
    o_ref, l_ref = _oracle(w, q, k, v)
    o, l = G.fwd_seq(w, q, k, v, fp32_check=False)
    G.assert_parity(o, l, o_ref, l_ref, fp32_check=False, what=f"small{case}, queued")


def _fwd(G, cfg, qd, kd, vd, n, stream=None):
    out = torch.full((qd.shape[0], n, qd.shape[2], qd.shape[3]), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((qd.shape[0], qd.shape[2], n), float("nan"), dtype=torch.float32, device="cuda")
    st = stream if stream is not None else torch.cuda.current_stream()
    G.sa.seg_attn_fwd_seq(cfg, qd, kd, vd, n, out, lse, st.cuda_stream)
    return out, lse


def test_item_queues_run_every_item_exactly_once(monkeypatch):
    """Queued or not, an item is the same arithmetic in the same order: over a few thousand items
    (more than fit the chip at once, so the order they are taken in varies) the two forms must
    agree bit for bit, on repeated launches (the counters are cleared in front of each), and a
    launch that has more workgroups than items must leave nothing unwritten."""
    import gpu_util as G
    w = W.small("queued", index=143, seq_len=6000, seg_len=1024, tail_len=256, n_q_heads=16, n_kv_heads=8,
                head_dim=128, kv_policy=[3, 1, 0, 3, 1, 1, 2, 0], batch=2)
    q, k, v = W.prefill_inputs(w)
    qd, kd, vd = G.dev_bf16(q), G.dev_bf16(k), G.dev_bf16(v)
    monkeypatch.setitem(G.TUNING, "item_queues", G.QUEUES_OFF)
    cfg = G.config_of(w, out_fp32=True, batch=2)
    o0, l0 = _fwd(G, cfg, qd, kd, vd, 6000)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(o0).all())
    monkeypatch.setitem(G.TUNING, "item_queues", G.QUEUES_ON_SMALL_GRID)
    cfg = G.config_of(w, out_fp32=True, batch=2)
    for _ in range(3):
        o1, l1 = _fwd(G, cfg, qd, kd, vd, 6000)
        torch.cuda.synchronize()
        assert torch.equal(o0, o1) and torch.equal(l0, l1)
    rows = np.array([0, 1023, 1024, 3071, 5999])
    o_ref, l_ref = _oracle(w, q, k, v, rows=rows)
    G.assert_parity(G.to_f64(o1)[:, rows], G.to_f64(l1)[:, :, rows], o_ref, l_ref, fp32_check=False, what="queued")


def test_item_queues_on_two_streams_do_not_share_counters(monkeypatch):
    """Launches on different streams may overlap: each stream has queue counters of its own, so
    two different problems in flight at once both come out as they do alone."""
    import gpu_util as G
    monkeypatch.setitem(G.TUNING, "item_queues", G.QUEUES_ON_SMALL_GRID)
    probs = []
    for i, n in enumerate((5000, 3333)):
        w = W.small(f"two{i}", index=144 + i, seq_len=n, seg_len=512, tail_len=128, n_q_heads=16, n_kv_heads=4,
                    head_dim=128, kv_policy=[3, 1, 1, 2])
        q, k, v = W.prefill_inputs(w)
        qd, kd, vd = G.dev_bf16(q), G.dev_bf16(k), G.dev_bf16(v)
        cfg = G.config_of(w, out_fp32=True, batch=1)
        alone = _fwd(G, cfg, qd, kd, vd, n)
        probs.append((cfg, qd, kd, vd, n, alone))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for _ in range(3):
        got = []
        for _rep in range(4):   # several launches per stream, interleaved on the host
            for (cfg, qd, kd, vd, n, _), s in zip(probs, streams):
                got.append(_fwd(G, cfg, qd, kd, vd, n, stream=s))
        torch.cuda.synchronize()
        for j, (o, l) in enumerate(got):
            o_a, l_a = probs[j % 2][5]
            assert torch.equal(o, o_a) and torch.equal(l, l_a)


def test_item_queues_with_two_host_threads_on_one_stream(monkeypatch):
    """Two host threads that launch into the same stream: every launch's counter reset and the
    launch itself must enter the stream as a pair, whatever the threads' timing."""
    import threading
    import gpu_util as G
    monkeypatch.setitem(G.TUNING, "item_queues", G.QUEUES_ON_SMALL_GRID)
    stream = torch.cuda.Stream()
    probs = []
    for i, n in enumerate((2100, 1500)):
        w = W.small(f"thr{i}", index=146 + i, seq_len=n, seg_len=512, tail_len=128, n_q_heads=8, n_kv_heads=2,
                    head_dim=128, kv_policy=[3, 1])
        q, k, v = W.prefill_inputs(w)
        qd, kd, vd = G.dev_bf16(q), G.dev_bf16(k), G.dev_bf16(v)
        cfg = G.config_of(w, out_fp32=True, batch=1)
        alone = _fwd(G, cfg, qd, kd, vd, n)
        outs = [(torch.empty_like(alone[0]), torch.empty_like(alone[1])) for _ in range(12)]
        probs.append((cfg, qd, kd, vd, n, alone, outs))
    torch.cuda.synchronize()
    errors = []

    def work(prob):
        cfg, qd, kd, vd, n, _, outs = prob
        try:
            for o, l in outs:
                G.sa.seg_attn_fwd_seq(cfg, qd, kd, vd, n, o, l, stream.cuda_stream)
        except Exception as e:   # noqa: BLE001 - reported below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(pr,)) for pr in probs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    stream.synchronize()
    assert not errors
    for _, _, _, _, _, alone, outs in probs:
        for o, l in outs:
            assert torch.equal(o, alone[0]) and torch.equal(l, alone[1])


_FIRST_CALLS_SCRIPT = r"""
import sys, threading
import numpy as np, torch
sys.path.insert(0, sys.argv[1]); sys.path.insert(0, sys.argv[1] + "/tests")
import workloads as W, gpu_util as G
G.TUNING["item_queues"] = G.QUEUES_ON_SMALL_GRID
torch.zeros(1, device="cuda")                       # the runtime is up; the library has launched nothing yet
probs = []
for i, n in enumerate((2300, 1700)):
    w = W.small(f"first{i}", index=170 + i, seq_len=n, seg_len=512, tail_len=128, n_q_heads=8, n_kv_heads=2,
                head_dim=128, kv_policy=[3, 1])
    q, k, v = W.prefill_inputs(w)
    qd, kd, vd = G.dev_bf16(q), G.dev_bf16(k), G.dev_bf16(v)
    cfg = G.config_of(w, out_fp32=True, batch=1)
    outs = [(torch.full((1, n, 8, 128), float("nan"), device="cuda"), torch.full((1, 8, n), float("nan"), device="cuda"))
            for _ in range(6)]
    probs.append((cfg, qd, kd, vd, n, outs, torch.cuda.Stream()))
torch.cuda.synchronize()
gate, errors = threading.Barrier(2), []
def work(pr):
    cfg, qd, kd, vd, n, outs, st = pr
    try:
        gate.wait()                                 # both threads make their first library call together
        for o, l in outs:
            G.sa.seg_attn_fwd_seq(cfg, qd, kd, vd, n, o, l, st.cuda_stream)
    except Exception as e:
        errors.append(repr(e))
ts = [threading.Thread(target=work, args=(pr,)) for pr in probs]
[t.start() for t in ts]; [t.join() for t in ts]
torch.cuda.synchronize()
assert not errors, errors
for cfg, qd, kd, vd, n, outs, st in probs:          # afterwards, one thread: the reference
    o_ref, l_ref = torch.empty_like(outs[0][0]), torch.empty_like(outs[0][1])
    G.sa.seg_attn_fwd_seq(cfg, qd, kd, vd, n, o_ref, l_ref, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(o_ref).all())
    for o, l in outs:
        assert torch.equal(o, o_ref) and torch.equal(l, l_ref)
print("first calls ok")
"""


def test_first_library_calls_from_two_host_threads():
    """A fresh process whose very first launches come from two host threads at once (same kernel
    instantiation, item queues on, a stream each): the one-time set-up of a kernel -- its LDS
    allowance, the resident-workgroup count, the queue counters' address -- must be safe to race
    through, and every launch must come out as it does later from one thread."""
    import subprocess
    import sys
    from conftest import ROOT
    res = subprocess.run([sys.executable, "-c", _FIRST_CALLS_SCRIPT, ROOT], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0 and "first calls ok" in res.stdout, res.stdout[-2000:] + res.stderr[-2000:]
