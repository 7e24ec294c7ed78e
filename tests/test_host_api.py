"""CPU-only checks of the C ABI: the library loads, exports every symbol the header
declares, and validates arguments before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2605_11744_amd as sa
from conftest import ROOT


def _header_symbols():
    text = open(os.path.join(ROOT, "include", "segattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(seg(?:attn)?_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = sa.lib()
    names = _header_symbols()
    assert len(names) >= 16
    for n in names:
        assert hasattr(L, n), n
    assert sorted(sa.EXPORTS) == names
    assert "gfx950" in sa.segattn_version()


def _cfg(**kw):
    base = dict(batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, seg_len=64, tail_len=16,
                kv_policy=[1, 3], past_capacity=256)
    base.update(kw)
    return sa.make_config(**base)


def test_cache_bytes_accounts_for_rows_counters_and_workspace():
    cfg = _cfg()
    total = sa.segattn_cache_bytes(cfg)
    kv_rows = 256 + (16 + 64)                      # PAST head: capacity; TAIL head: T + S
    kv_bytes = kv_rows * 2 * 128 * 2
    assert kv_bytes < total < kv_bytes + 64 * 1024
    assert sa.segattn_cache_bytes(_cfg(batch=3)) > 3 * kv_bytes
    # a pool that can hold prefixes worth cutting into pieces (>= 1024 rows each) adds the
    # split-prefix workspace: fp32 output rows + LSEs of one segment per piece, at most 4 pieces
    big = _cfg(seg_len=512, tail_len=64, past_capacity=8192)
    kv_big = (8192 + (64 + 512)) * 2 * 128 * 2
    ws = 4 * 512 * 4 * (128 + 1) * 4               # pieces x S x (1 PAST head x g = 4 heads) x (D + 1) floats
    assert kv_big + ws < sa.segattn_cache_bytes(big) < kv_big + ws + 256 * 1024
    assert sa.segattn_cache_bytes(_cfg(seg_len=512, tail_len=64, past_capacity=8192, batch=64)) < 64 * (kv_big + 256 * 1024)


@pytest.mark.parametrize("bad", [
    dict(head_dim=96), dict(n_q_heads=7), dict(tail_len=65), dict(seg_len=0), dict(batch=0),
    dict(kv_policy=[1, 4]), dict(past_capacity=32), dict(tail_len=-1), dict(scale=-1.0),
    dict(n_kv_heads=0, n_q_heads=0, kv_policy=[]), dict(rope_theta=-1.0),
    dict(prefill_waves=2), dict(prefill_waves=-8), dict(item_queues=4), dict(item_queues=-1),
])
def test_invalid_configurations_are_rejected(bad):
    cfg = _cfg(**bad)
    assert sa.segattn_cache_bytes(cfg) == 0
    with pytest.raises(sa.SegattnError) as e:
        sa.segattn_create(cfg, 256, 1 << 30)
    assert e.value.status == sa.SEGATTN_EINVAL


def test_create_checks_arena_and_calls_check_state_and_pointers():
    cfg = _cfg()
    need = sa.segattn_cache_bytes(cfg)
    with pytest.raises(sa.SegattnError):
        sa.segattn_create(cfg, 0, need)                 # null arena
    with pytest.raises(sa.SegattnError):
        sa.segattn_create(cfg, 4096 + 8, need)          # misaligned
    with pytest.raises(sa.SegattnError):
        sa.segattn_create(cfg, 4096, need - 1)          # too small
    ctx = sa.segattn_create(cfg, 4096, need)            # create touches no device memory
    try:
        with pytest.raises(sa.SegattnError) as e:       # nothing reset yet
            sa.seg_attn_fwd(ctx, 4096, 4096, 4096, 8, 4096, 4096)
        assert e.value.status == sa.SEGATTN_ESTATE
        with pytest.raises(sa.SegattnError) as e:
            sa.seg_attn_fwd(ctx, 0, 4096, 4096, 8, 4096, 4096)
        assert e.value.status == sa.SEGATTN_EINVAL
        with pytest.raises(sa.SegattnError) as e:
            sa.seg_kv_past_append(ctx, 0, 4096, 4096, 4)    # head 0 is not PAST
        assert e.value.status == sa.SEGATTN_EINVAL
        with pytest.raises(sa.SegattnError) as e:
            sa.seg_kv_set_lengths(ctx, [65], [0], [0])      # not a multiple of S
        assert e.value.status == sa.SEGATTN_EINVAL
        with pytest.raises(sa.SegattnError) as e:
            sa.seg_kv_set_lengths(ctx, [512], [16], [0])    # beyond the pool capacity
        assert e.value.status == sa.SEGATTN_ECAPACITY
        assert sa.segattn_cache_span(ctx, 0, 1)[2] == 256 and sa.segattn_cache_span(ctx, 0, 0)[2] == 80
        with pytest.raises(sa.SegattnError):
            sa.segattn_cache_span(ctx, 1, 0)
        assert sa.segattn_resident_bytes(ctx) == 0
    finally:
        sa.segattn_destroy(ctx)


def test_retrieval_mode_configuration_and_select_validation():
    """Retrieval mode (retrieved_capacity > 0): needs a PAST head, forbids TAIL|PAST, adds the
    attention views to the arena; seg_kv_past_select checks mode, size and pool contents."""
    plain = sa.segattn_cache_bytes(_cfg(kv_policy=[1, 2]))
    with_views = sa.segattn_cache_bytes(_cfg(kv_policy=[1, 2], retrieved_capacity=32))
    view_bytes = 2 * (32 + 64) * 128 * 2          # one PAST head: K and V of R_max + S rows
    assert plain > 0 and view_bytes <= with_views - plain < view_bytes + 4096
    for bad in (dict(kv_policy=[1, 3], retrieved_capacity=32), dict(kv_policy=[1, 0], retrieved_capacity=32),
                dict(kv_policy=[1, 2], retrieved_capacity=-1)):
        assert sa.segattn_cache_bytes(_cfg(**bad)) == 0
    cfg = _cfg(kv_policy=[1, 2], retrieved_capacity=32)
    ctx = sa.segattn_create(cfg, 4096, sa.segattn_cache_bytes(cfg))
    try:
        with pytest.raises(sa.SegattnError) as e:
            sa.seg_kv_past_select(ctx, 4096, 4)             # nothing reset yet
        assert e.value.status == sa.SEGATTN_ESTATE
        with pytest.raises(sa.SegattnError) as e:
            sa.seg_kv_past_select(ctx, 4096, 33)            # beyond retrieved_capacity
        assert e.value.status == sa.SEGATTN_EINVAL
        with pytest.raises(sa.SegattnError) as e:
            sa.seg_kv_past_select(ctx, 0, 4)                # null list
        assert e.value.status == sa.SEGATTN_EINVAL
        with pytest.raises(sa.SegattnError) as e:
            sa.seg_kv_set_lengths(ctx, [64], [16], [3])     # open segment cannot be declared here
        assert e.value.status == sa.SEGATTN_EINVAL
    finally:
        sa.segattn_destroy(ctx)
    ctx = sa.segattn_create(_cfg(), 4096, sa.segattn_cache_bytes(_cfg()))
    try:
        with pytest.raises(sa.SegattnError) as e:
            sa.seg_kv_past_select(ctx, 4096, 4)             # context is not in retrieval mode
        assert e.value.status == sa.SEGATTN_EINVAL
    finally:
        sa.segattn_destroy(ctx)


def test_fwd_seq_validates_before_launching():
    cfg = _cfg()
    with pytest.raises(sa.SegattnError) as e:
        sa.seg_attn_fwd_seq(cfg, 4096, 4096, 0, 128, 4096, 4096)
    assert e.value.status == sa.SEGATTN_EINVAL
    with pytest.raises(sa.SegattnError) as e:
        sa.seg_attn_fwd_seq(cfg, 4096, 4096, 4096, 0, 4096, 4096)
    assert e.value.status == sa.SEGATTN_EINVAL
    assert sa.strerror(sa.SEGATTN_ECAPACITY).startswith("past pool")


def test_probes_validate_before_touching_a_device():
    with pytest.raises(sa.SegattnError) as e:
        sa.segattn_bandwidth_probe(4096, 1 << 20, 2, 4096)          # no such mode
    assert e.value.status == sa.SEGATTN_EINVAL
    with pytest.raises(sa.SegattnError) as e:
        sa.segattn_bandwidth_probe(4096 + 8, 1 << 20, 0, 4096)      # misaligned
    assert e.value.status == sa.SEGATTN_EINVAL
    for iters, sink in ((0, 4096), (10_000_001, 4096), (1000, 0), (1000, 4096 + 2)):
        with pytest.raises(sa.SegattnError) as e:
            sa.segattn_mfma_probe(iters, sink)
        assert e.value.status == sa.SEGATTN_EINVAL
    for us, counts in ((0, 4096), (10_000_001, 4096), (1000, 0), (1000, 4096 + 4)):
        with pytest.raises(sa.SegattnError) as e:
            sa.segattn_clock_probe(us, counts)
        assert e.value.status == sa.SEGATTN_EINVAL


def test_layer_policy_follows_the_head_and_layer_sets():
    """Sec. 3.4: local heads carry the tail in every layer; long-range heads read the past in the
    layers of L_long and only their own segment elsewhere."""
    assert sa.segattn_layer_policy(8, [0, 5], True) == [2, 1, 1, 1, 1, 2, 1, 1]
    assert sa.segattn_layer_policy(8, [0, 5], False) == [0, 1, 1, 1, 1, 0, 1, 1]
    assert sa.segattn_layer_policy(4, [], True) == [1, 1, 1, 1]
    with pytest.raises(sa.SegattnError):
        sa.segattn_layer_policy(4, [4], True)
