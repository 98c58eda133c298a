"""Host-side checks that need no GPU: the library loads, exports every declared
symbol, sizes follow Eq. 2, and the per-layer state machine of Alg. 1 rejects
bad calls without touching the device (dry-run caches enqueue nothing)."""
import ctypes

import pytest

import paper_2604_16734_amd as K
from kvp_workload import WORKLOADS, get_workload, chunk_ranges
from oracle import kvp_oracle as O


def _cfg(wl, merge=1, sets=1, flags=K.KVP_FLAG_DRY_RUN, **over):
    c = K.KvpConfig(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.budget, wl.chunk,
                    merge, sets, flags, 0.0)
    for k, v in over.items():
        setattr(c, k, v)
    return c


def test_library_exports_every_declared_symbol():
    L = K.lib()
    names = K.declared_symbols()
    assert {"kvp_init_cache", "kvp_prefill_chunk", "kvp_compact", "kvp_decode_ready"} <= set(names)
    for name in names:
        assert hasattr(L, name), name


def test_strerror_and_kernel_names():
    assert K.kvp_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert K.kvp_strerror(code)
    assert [K.kvp_kernel_name(i) for i in range(len(K.KERNEL_KINDS))] == list(K.KERNEL_KINDS)


def test_persistent_bytes_follow_eq2():
    # Eq. 2 at sequence length M, bf16, plus 8 bytes of metadata per slot
    for wl in WORKLOADS:
        cfg = _cfg(wl)
        kv = O.kv_cache_bytes(wl.n_layers, wl.n_kv_heads, wl.head_dim, 2, wl.budget)
        meta = 8 * wl.n_layers * wl.n_kv_heads * wl.budget
        assert K.kvp_persistent_bytes(cfg) == kv + meta
        total = K.kvp_cache_bytes(cfg)
        assert total > kv + meta
        # two scratch sets cost exactly one more set
        total2 = K.kvp_cache_bytes(_cfg(wl, sets=2 if wl.n_layers > 1 else 1))
        assert total2 >= total


@pytest.mark.parametrize("field,value", [
    ("n_layers", 0), ("n_q_heads", 5), ("n_kv_heads", 0), ("head_dim", 96), ("budget", 0),
    ("chunk_max", 0), ("merge", 2), ("scratch_sets", -1), ("flags", 8), ("softmax_scale", -1.0),
    ("budget", 8190),
])
def test_invalid_config_rejected(field, value):
    wl = get_workload("tiny")
    cfg = _cfg(wl, **{field: value})
    assert K.kvp_cache_bytes(cfg) == 0
    rc, h = K.kvp_init_cache(cfg, wl.segments, None, 0)
    assert rc == K.KVP_EINVAL and not h


def test_segment_validation():
    wl = get_workload("tiny")
    cfg = _cfg(wl)
    S = K.KvpSegment
    bad = [
        [S(0, 10, 1, 2, 5, 1, 0), S(11, 5, 0, 0, 0, 0, 0)],      # gap
        [S(1, 10, 0, 0, 0, 0, 0)],                               # does not start at 0
        [S(0, 10, 1, 3, 3, 1, 0)],                               # 3*3*1 != 10
        [S(0, 10, 2, 0, 0, 0, 0)],                               # unknown kind
        [S(0, 0, 0, 0, 0, 0, 0)],                                # empty
        [S(0, 8, 1, 2, 2, 2, 5)],                                # temporal flag
    ]
    for segs in bad:
        rc, h = K.kvp_init_cache(cfg, segs, None, 0)
        assert rc == K.KVP_EINVAL and not h
    rc, h = K.kvp_init_cache(cfg, [], None, 0)
    assert rc == K.KVP_EINVAL


def test_device_buffer_checks_without_dry_run():
    wl = get_workload("tiny")
    cfg = _cfg(wl, flags=0)
    need = K.kvp_cache_bytes(cfg)
    rc, h = K.kvp_init_cache(cfg, wl.segments, None, need)            # null buffer
    assert rc == K.KVP_EINVAL and not h
    rc, h = K.kvp_init_cache(cfg, wl.segments, 4096 + 8, need)        # misaligned
    assert rc == K.KVP_EINVAL and not h
    rc, h = K.kvp_init_cache(cfg, wl.segments, 4096, need - 1)        # too small
    assert rc == K.KVP_ENOMEM and not h


def test_state_machine_and_counts():
    wl = get_workload("tiled_image")
    cfg = _cfg(wl)
    rc, h = K.kvp_init_cache(cfg, wl.segments, None, 0)
    assert rc == K.KVP_OK and h
    try:
        # compact before any block, and decode view of an empty layer
        assert K.kvp_compact(h, 0) == K.KVP_ESTATE
        rc, vw = K.kvp_decode_ready(h, 0)
        assert rc == K.KVP_OK and vw.count == 0 and vw.budget == wl.budget and vw.next_token == 0
        # bad layer / sizes / order
        assert K.kvp_prefill_chunk(h, wl.n_layers, 0, 8, 0, 0, 0, 0) == K.KVP_EINVAL
        assert K.kvp_prefill_chunk(h, -1, 0, 8, 0, 0, 0, 0) == K.KVP_EINVAL
        assert K.kvp_prefill_chunk(h, 0, 0, 0, 0, 0, 0, 0) == K.KVP_EINVAL
        assert K.kvp_prefill_chunk(h, 0, 0, wl.chunk + 1, 0, 0, 0, 0) == K.KVP_EINVAL
        assert K.kvp_prefill_chunk(h, 0, 5, 8, 0, 0, 0, 0) == K.KVP_ESTATE          # tokens skipped
        # the whole prefix, counts follow min(M, c + n) (Alg. 1 lines 8-11)
        count = 0
        for t0, n in chunk_ranges(wl.n_tokens, wl.chunk):
            for layer in range(wl.n_layers):
                assert K.kvp_prefill_chunk(h, layer, t0, n, 0, 0, 0, 0) == K.KVP_OK
                assert K.kvp_prefill_chunk(h, layer, t0 + n, 1, 0, 0, 0, 0) == K.KVP_ESTATE   # pending
                rc, _ = K.kvp_decode_ready(h, layer)
                assert rc == K.KVP_ESTATE
                assert K.kvp_compact(h, layer) == K.KVP_OK
                assert K.kvp_compact(h, layer) == K.KVP_ESTATE
                rc, vw = K.kvp_decode_ready(h, layer)
                assert rc == K.KVP_OK and vw.count == min(wl.budget, count + n) and vw.next_token == t0 + n
            count = min(wl.budget, count + n)
        # past the end of the prefix
        assert K.kvp_prefill_chunk(h, 0, wl.n_tokens, 1, 0, 0, 0, 0) == K.KVP_EINVAL
        # restore
        assert K.kvp_set_state(h, 0, wl.budget + 1, 10) == K.KVP_EINVAL
        assert K.kvp_set_state(h, 0, 10, 5) == K.KVP_EINVAL
        assert K.kvp_set_state(h, 0, 100, 300) == K.KVP_OK
        rc, vw = K.kvp_decode_ready(h, 0)
        assert vw.count == 100 and vw.next_token == 300
        assert K.kvp_prefill_chunk(h, 0, 300, 16, 0, 0, 0, 0) == K.KVP_OK
    finally:
        K.kvp_free_cache(h)


def test_proxy_and_keydiff_entry_points_follow_the_same_state_machine():
    wl = get_workload("tiny")
    cfg = _cfg(wl)
    rc, h = K.kvp_init_cache(cfg, wl.segments, None, 0)
    assert rc == K.KVP_OK and h
    try:
        assert K.kvp_prefill_chunk_proxy(h, 0, 0, 8, 0, 0, 0, 0, 0, 0) == K.KVP_EINVAL            # no proxy rows
        assert K.kvp_prefill_chunk_proxy(h, 0, 0, 8, 0, 0, 0, 0, 0, wl.chunk + 1) == K.KVP_EINVAL  # too many
        assert K.kvp_prefill_chunk_proxy(h, 0, 3, 8, 0, 0, 0, 0, 0, 4) == K.KVP_ESTATE            # tokens skipped
        count = 0
        for t0, n in chunk_ranges(wl.n_tokens, wl.chunk):
            if (t0 // wl.chunk) % 2:
                assert K.kvp_prefill_chunk_proxy(h, 0, t0, n, 0, 0, 0, 0, 0, 4) == K.KVP_OK
            else:
                assert K.kvp_prefill_chunk_keydiff(h, 0, t0, n, 0, 0, 0, 0) == K.KVP_OK
            assert K.kvp_prefill_chunk(h, 0, t0 + n, 1, 0, 0, 0, 0) == K.KVP_ESTATE               # pending
            assert K.kvp_compact(h, 0) == K.KVP_OK
            count = min(wl.budget, count + n)
            rc, vw = K.kvp_decode_ready(h, 0)
            assert rc == K.KVP_OK and vw.count == count and vw.next_token == t0 + n
    finally:
        K.kvp_free_cache(h)


def test_decode_step_state_machine():
    wl = get_workload("single_image")
    rc, h = K.kvp_init_cache(_cfg(wl, sets=2), wl.segments, None, 0)
    assert rc == K.KVP_OK
    try:
        assert K.kvp_decode_step(h, 0, 0, 0, 0, 1, 0) == K.KVP_OK                # an empty cache: the tail alone
        assert K.kvp_decode_step(h, 0, 0, 0, 0, 0, 0) == K.KVP_EINVAL            # no current token
        assert K.kvp_decode_step(h, 0, 0, 0, 0, (1 << 20) + 1, 0) == K.KVP_EINVAL
        assert K.kvp_decode_step(h, wl.n_layers, 0, 0, 0, 1, 0) == K.KVP_EINVAL
        assert K.kvp_prefill_chunk(h, 0, 0, 16, 0, 0, 0, 0) == K.KVP_OK
        assert K.kvp_decode_step(h, 0, 0, 0, 0, 1, 0) == K.KVP_ESTATE            # the layer is pending
        assert K.kvp_decode_step(h, 2, 0, 0, 0, 1, 0) == K.KVP_ESTATE            # its scratch set is taken
        assert K.kvp_decode_step(h, 1, 0, 0, 0, 1, 0) == K.KVP_OK                # the other set is free
        assert K.kvp_compact(h, 0) == K.KVP_OK
        rc, before = K.kvp_decode_ready(h, 0)
        assert K.kvp_decode_step(h, 0, 0, 0, 0, 3, 0) == K.KVP_OK
        rc, after = K.kvp_decode_ready(h, 0)
        assert (after.count, after.next_token) == (before.count, before.next_token) == (16, 16)
    finally:
        K.kvp_free_cache(h)


def test_static_scratch_decode_step_limits():
    """kvp_decode_step_static refuses a step whose partial results do not fit its 1 MiB array with
    at least 16 workgroups per KV head (or all it wants, if fewer), and follows the state machine
    of kvp_decode_step except that a taken scratch set does not matter."""
    from kvp_workload import Segment, Workload
    segs = (Segment(0, 4096, 0),)
    fits = Workload("fits", 2, 64, 8, 128, 64, 1024, segs)          # 64 heads x 130 floats x 16 = 133120 floats
    too_big = Workload("too_big", 2, 128, 8, 128, 64, 1024, segs)   # 128 heads: only 15 sets of partials fit
    for wl, many_keys_rc in ((fits, K.KVP_OK), (too_big, K.KVP_ENOMEM)):
        rc, h = K.kvp_init_cache(_cfg(wl), wl.segments, None, 0)
        assert rc == K.KVP_OK
        try:
            assert K.kvp_decode_step_static(h, 0, 0, 0, 0, 1, 0) == K.KVP_OK           # one key: one workgroup is all it wants
            assert K.kvp_decode_step_static(h, 0, 0, 0, 0, 0, 0) == K.KVP_EINVAL
            assert K.kvp_decode_step_static(h, 9, 0, 0, 0, 1, 0) == K.KVP_EINVAL
            assert K.kvp_set_state(h, 0, 1024, 1024) == K.KVP_OK
            assert K.kvp_decode_step_static(h, 0, 0, 0, 0, 1, 0) == many_keys_rc       # 17 workgroups wanted
            assert K.kvp_decode_step(h, 0, 0, 0, 0, 1, 0) == K.KVP_OK                  # the scratch set is roomier
            assert K.kvp_prefill_chunk(h, 1, 0, 16, 0, 0, 0, 0) == K.KVP_OK            # layer 1 pending, set taken
            assert K.kvp_decode_step_static(h, 1, 0, 0, 0, 1, 0) == K.KVP_ESTATE
            assert K.kvp_decode_step(h, 0, 0, 0, 0, 1, 0) == K.KVP_ESTATE
            assert K.kvp_decode_step_static(h, 0, 0, 0, 0, 1, 0) == many_keys_rc
        finally:
            K.kvp_free_cache(h)


def test_prefill_block_walks_every_layer():
    """kvp_prefill_block in a dry run (no device work, so everything on one stream): every layer
    advances by the block, errors are reported before any layer moves, and a per-layer call that
    leaves a layer pending makes the block call stop at that layer with the earlier ones done."""
    wl = get_workload("tiled_image")
    rc, h = K.kvp_init_cache(_cfg(wl, sets=wl.n_layers), wl.segments, None, 0)    # a scratch set per layer
    assert rc == K.KVP_OK
    zeros = [0] * wl.n_layers
    try:
        assert K.kvp_prefill_block(h, 0, wl.chunk + 1, zeros, zeros, zeros, zeros) == K.KVP_EINVAL
        assert K.kvp_prefill_block(h, 5, 8, zeros, zeros, zeros, zeros) == K.KVP_ESTATE          # tokens skipped
        assert K.kvp_prefill_block(h, 0, 8, zeros, zeros, zeros, zeros, scoring=7) == K.KVP_EINVAL
        assert K.kvp_prefill_block(h, 0, 8, zeros, zeros, zeros, zeros, scoring=K.KVP_SCORE_PROXY) == K.KVP_EINVAL  # no proxy queries
        for layer in range(wl.n_layers):
            rc, vw = K.kvp_decode_ready(h, layer)
            assert rc == K.KVP_OK and (vw.count, vw.next_token) == (0, 0)
        t = 0
        for n, scoring in ((wl.chunk, K.KVP_SCORE_OWN), (wl.chunk, K.KVP_SCORE_KEYDIFF), (40, K.KVP_SCORE_PROXY)):
            obs = zeros if scoring == K.KVP_SCORE_PROXY else None
            assert K.kvp_prefill_block(h, t, n, zeros, zeros, zeros, zeros, scoring=scoring, q_obs=obs, n_obs=4) == K.KVP_OK
            t += n
            for layer in range(wl.n_layers):
                rc, vw = K.kvp_decode_ready(h, layer)
                assert rc == K.KVP_OK and (vw.count, vw.next_token) == (min(wl.budget, t), t)
        assert K.kvp_prefill_join(h) == K.KVP_OK
        # layer 3 taken out of step by a per-layer call: the block call does layers 0-2 and stops there
        assert K.kvp_prefill_chunk(h, 3, t, 8, 0, 0, 0, 0) == K.KVP_OK
        assert K.kvp_prefill_block(h, t, 8, zeros, zeros, zeros, zeros) == K.KVP_ESTATE
        for layer in range(wl.n_layers):
            rc, vw = K.kvp_decode_ready(h, layer)
            if layer < 3:
                assert rc == K.KVP_OK and vw.next_token == t + 8
            elif layer == 3:
                assert rc == K.KVP_ESTATE
            else:
                assert rc == K.KVP_OK and vw.next_token == t
    finally:
        K.kvp_free_cache(h)


def test_compact_layers_state_machine():
    """kvp_compact_layers in a dry run: a range of PENDING layers becomes READY with the block
    appended; a range that holds a layer that is not PENDING, or that is out of bounds, is refused
    with nothing changed; layers out of step with one another are still all compacted."""
    wl = get_workload("tiled_image")
    rc, h = K.kvp_init_cache(_cfg(wl, sets=wl.n_layers), wl.segments, None, 0)
    assert rc == K.KVP_OK
    try:
        nl = wl.n_layers
        assert K.kvp_compact_layers(None, 0, 1) == K.KVP_EINVAL
        for first, count in ((-1, 2), (0, 0), (0, nl + 1), (nl - 1, 2), (nl, 1)):
            assert K.kvp_compact_layers(h, first, count) == K.KVP_EINVAL
        assert K.kvp_compact_layers(h, 0, nl) == K.KVP_ESTATE                 # nothing pending
        for layer in range(nl - 1):
            assert K.kvp_prefill_chunk(h, layer, 0, 24, 0, 0, 0, 0) == K.KVP_OK
        assert K.kvp_compact_layers(h, 0, nl) == K.KVP_ESTATE                 # the last layer is READY
        for layer in range(nl - 1):
            assert K.kvp_decode_ready(h, layer)[0] == K.KVP_ESTATE            # still pending, all of them
        assert K.kvp_compact_layers(h, 0, nl - 1) == K.KVP_OK
        for layer in range(nl):
            rc, vw = K.kvp_decode_ready(h, layer)
            assert rc == K.KVP_OK and (vw.count, vw.next_token) == ((24, 24) if layer < nl - 1 else (0, 0))
        # layers out of step with one another (the last one is a block behind): still one call
        assert K.kvp_prefill_chunk(h, nl - 1, 0, 24, 0, 0, 0, 0) == K.KVP_OK
        for layer in range(nl - 1):
            assert K.kvp_prefill_chunk(h, layer, 24, 8, 0, 0, 0, 0) == K.KVP_OK
        assert K.kvp_compact_layers(h, 0, nl) == K.KVP_OK
        for layer in range(nl):
            rc, vw = K.kvp_decode_ready(h, layer)
            assert rc == K.KVP_OK and vw.next_token == (32 if layer < nl - 1 else 24)
        assert K.kvp_compact_layers(h, 2, 3) == K.KVP_ESTATE
        # scoring passes put off until the compaction: the per-layer calls and both ways of compacting
        assert K.kvp_set_deferred_scoring(None, 1) == K.KVP_EINVAL
        assert K.kvp_set_deferred_scoring(h, 2) == K.KVP_EINVAL
        assert K.kvp_set_deferred_scoring(h, 1) == K.KVP_OK
        t = 32                                     # every layer but the last stands at token 32
        assert K.kvp_prefill_chunk(h, nl - 1, 24, 8, 0, 0, 0, 0) == K.KVP_OK
        assert K.kvp_compact(h, nl - 1) == K.KVP_OK
        while t < wl.budget + 2 * wl.chunk:        # well into the blocks that evict
            for layer in range(nl):
                if layer % 2:
                    assert K.kvp_prefill_chunk_keydiff(h, layer, t, wl.chunk, 0, 0, 0, 0) == K.KVP_OK
                else:
                    assert K.kvp_prefill_chunk_proxy(h, layer, t, wl.chunk, 0, 0, 0, 0, 0, 8) == K.KVP_OK
            assert K.kvp_compact(h, 0) == K.KVP_OK
            assert K.kvp_compact_layers(h, 1, nl - 1) == K.KVP_OK
            t += wl.chunk
            for layer in range(nl):
                rc, vw = K.kvp_decode_ready(h, layer)
                assert rc == K.KVP_OK and (vw.count, vw.next_token) == (min(wl.budget, t), t)
        assert K.kvp_set_deferred_scoring(h, 0) == K.KVP_OK
    finally:
        K.kvp_free_cache(h)


def test_scratch_sets_gate_pending_layers():
    wl = get_workload("single_image")
    for sets, second_ok in ((1, False), (2, True)):
        rc, h = K.kvp_init_cache(_cfg(wl, sets=sets), wl.segments, None, 0)
        assert rc == K.KVP_OK
        try:
            assert K.kvp_prefill_chunk(h, 0, 0, 16, 0, 0, 0, 0) == K.KVP_OK
            rc = K.kvp_prefill_chunk(h, 1, 0, 16, 0, 0, 0, 0)
            assert rc == (K.KVP_OK if second_ok else K.KVP_ESTATE)
            # layer 2 shares set 0 with layer 0 when there are two sets
            assert K.kvp_prefill_chunk(h, 2, 0, 16, 0, 0, 0, 0) == K.KVP_ESTATE
            assert K.kvp_compact(h, 0) == K.KVP_OK
            assert K.kvp_prefill_chunk(h, 2, 0, 16, 0, 0, 0, 0) == K.KVP_OK
        finally:
            K.kvp_free_cache(h)


def test_null_handles():
    assert K.kvp_compact(None, 0) == K.KVP_EINVAL
    assert K.kvp_prefill_chunk(None, 0, 0, 1, 0, 0, 0, 0) == K.KVP_EINVAL
    rc, _ = K.kvp_decode_ready(None, 0)
    assert rc == K.KVP_EINVAL
    K.kvp_free_cache(None)
    # Every cache this file creates is a dry run or is refused by validation: no call here may
    # reach a kernel launch, so no device pointer is ever made up for a cache that would use it.
    # "A real cache refuses null tensors before launching anything" is checked on a live
    # allocation in tests/test_gpu_parity.py::test_real_cache_refuses_null_tensors.
