"""Pins of the CPU oracle against things other than itself.

Each test names what fixes the expected value: an equation of the paper, a
closed form, a library routine, brute force, or an invariant of Alg. 1.  The
merge rules are this build's own (the paper is eviction-only); their fixtures
are worked by hand from rules M1-M5 stated in the oracle's header.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest
import torch

from kvp_workload import Segment, WORKLOADS, get_workload, layer_inputs, bf16_bits_to_f32, chunk_ranges
from oracle import kvp_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_bf16(rng, shape, scale=1.0):
    x = (scale * rng.standard_normal(shape)).astype(np.float32)
    u = x.view(np.uint32)
    u = ((u + ((u >> 16) & 1) + 0x7FFF) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


# ---------------------------------------------------------------- bf16 rounding
def test_round_to_bf16_matches_library_and_ties():
    # torch's float64 -> bfloat16 conversion is a library routine for the same rounding
    rng = np.random.default_rng(1)
    x = rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_to_bf16(x), want)
    # exact ties go to the even mantissa: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -7 + 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # one rounding, not two: just above a tie must go up even though the float32
    # rounding of the same number lands exactly on the tie
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert O.round_to_bf16(np.array([x]))[0] == 1.0 + 2.0 ** -7
    assert O.round_to_bf16(np.array([-x]))[0] == -(1.0 + 2.0 ** -7)
    assert O.round_to_bf16(np.array([0.0]))[0] == 0.0


def test_bf16_bits_roundtrip():
    bits = np.arange(0x3F00, 0x4100, dtype=np.uint16)
    assert np.array_equal(O.f64_to_bf16_bits(O.bf16_bits_to_f64(bits)), bits)


def test_bf16_bit_helpers_against_the_format_and_a_library_view():
    """Every finite bfloat16 pattern (both signs, zeros, subnormals, the largest finite value):
    the value must be what torch reads out of the same 16 bits, and what the format's definition
    gives, (-1)^s 2^(e-127) (1 + m/128), or (-1)^s 2^-126 (m/128) for e = 0; and the way back must
    return the same 16 bits."""
    bits = np.arange(1 << 16, dtype=np.uint32)
    e, m, sgn = (bits >> 7) & 0xFF, bits & 0x7F, np.where(bits >> 15, -1.0, 1.0)
    finite = e != 0xFF
    bits, e, m, sgn = bits[finite].astype(np.uint16), e[finite], m[finite], sgn[finite]
    assert len(bits) == 65536 - 256
    got = O.bf16_bits_to_f64(bits)
    by_library = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, by_library) and np.array_equal(np.signbit(got), np.signbit(by_library))
    by_definition = sgn * np.where(e == 0, np.ldexp(m / 128.0, -126), np.ldexp(1.0 + m / 128.0, e.astype(np.int64) - 127))
    assert np.array_equal(got, by_definition)
    # spot values nobody computes: 0x3F80 is 1, 0xC000 is -2, 0x3DCD is the bf16 next to 0.1, 0x7F7F the largest
    assert O.bf16_bits_to_f64(np.array([0x3F80, 0xC000, 0x0000, 0x7F7F], dtype=np.uint16)).tolist() == \
        [1.0, -2.0, 0.0, (2.0 - 2.0 ** -7) * 2.0 ** 127]
    assert abs(O.bf16_bits_to_f64(np.array([0x3DCD], dtype=np.uint16))[0] - 0.1) < 0.1 * 2.0 ** -8
    # the way back: the same bits, the sign of zero included
    back = O.f64_to_bf16_bits(by_library)
    assert back.dtype == np.uint16 and np.array_equal(back, bits)
    by_library_back = torch.from_numpy(by_library).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(back, by_library_back)
    # values that are not bfloat16 numbers are refused, not rounded
    for bad in (1.0 + 2.0 ** -8, 0.1, 1e-50, 1e39):
        with pytest.raises(ValueError):
            O.f64_to_bf16_bits(np.array([bad]))


# ---------------------------------------------------------------- Eq. 2
def test_kv_bytes_closed_form():
    # Eq. 2 at the budget, bf16: the persistent KV sizes of the five shapes
    want = {"tiny": 131072, "single_image": 16 << 20, "tiled_image": 8 << 20,
            "video": 32 << 20, "long_video": 256 << 20}
    full = {"tiny": 622592, "long_video": 2080 << 20}
    for w in WORKLOADS:
        assert O.kv_cache_bytes(w.n_layers, w.n_kv_heads, w.head_dim, 2, w.budget) == want[w.name]
        if w.name in full:
            assert O.kv_cache_bytes(w.n_layers, w.n_kv_heads, w.head_dim, 2, w.n_tokens) == full[w.name]


# ---------------------------------------------------------------- Eq. 1 / Eq. 4, brute force
def _brute_attend(q, k_all, v_all, c):
    n, hq, d = q.shape
    hkv, tot, _ = k_all.shape
    g = hq // hkv
    out = np.zeros((n, hq, d))
    scores = np.zeros((hkv, tot))
    for h in range(hq):
        hk = h // g
        for r in range(n):
            logits = []
            for j in range(tot):
                visible = j < c or (j - c) <= r
                if visible:
                    dot = 0.0
                    for e in range(d):
                        dot += q[r, h, e] * k_all[hk, j, e]
                    logits.append(dot / math.sqrt(d))
                else:
                    logits.append(None)
            mx = max(l for l in logits if l is not None)
            ex = [math.exp(l - mx) if l is not None else 0.0 for l in logits]
            z = sum(ex)
            for j in range(tot):
                pj = ex[j] / z
                scores[hk, j] += pj
                for e in range(d):
                    out[r, h, e] += pj * v_all[hk, j, e]
    return out, scores


@pytest.mark.parametrize("hq,hkv,c,n,d", [(2, 2, 0, 5, 4), (4, 2, 3, 6, 8), (3, 1, 7, 1, 4)])
def test_attend_chunk_brute_force(hq, hkv, c, n, d):
    rng = np.random.default_rng(hq * 100 + c)
    q = _rand_bf16(rng, (n, hq, d))
    k_all = _rand_bf16(rng, (hkv, c + n, d))
    v_all = _rand_bf16(rng, (hkv, c + n, d))
    out, scores = O.attend_chunk(q, k_all, v_all, c)
    bout, bscores = _brute_attend(q, k_all, v_all, c)
    np.testing.assert_allclose(out, bout, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(scores, bscores, rtol=1e-12, atol=1e-13)


def test_attend_chunk_closed_forms():
    # all keys equal: softmax is uniform over the visible keys, so row r of an
    # empty-cache block averages values 0..r and column j collects sum_{r>=j} 1/(r+1)
    n, d = 6, 4
    q = np.ones((n, 1, d))
    k_all = np.ones((1, n, d))
    v_all = np.arange(n, dtype=np.float64)[None, :, None] * np.ones((1, n, d))
    out, scores = O.attend_chunk(q, k_all, v_all, 0)
    for r in range(n):
        assert np.allclose(out[r, 0], r / 2.0)
    want = [sum(1.0 / (r + 1) for r in range(j, n)) for j in range(n)]
    np.testing.assert_allclose(scores[0], want, rtol=1e-13)
    # one key dominating by a known margin: two keys, logits (a, 0) -> weights sigmoid(a)
    a = 3.0
    q = np.array([[[2.0, 0.0, 0.0, 0.0]]])
    k_all = np.array([[[a, 0, 0, 0], [0, 0, 0, 0]]], dtype=np.float64)      # scale 1/2, logit a
    v_all = np.array([[[1.0, 0, 0, 0], [0, 1.0, 0, 0]]])
    out, scores = O.attend_chunk(q, k_all, v_all, 1)
    s = 1.0 / (1.0 + math.exp(-a))
    np.testing.assert_allclose(out[0, 0], [s, 1 - s, 0, 0], rtol=1e-13)
    np.testing.assert_allclose(scores[0], [s, 1 - s], rtol=1e-13)
    # an explicit scale is honoured
    out2, _ = O.attend_chunk(q, k_all, v_all, 1, scale=1.0)
    s2 = 1.0 / (1.0 + math.exp(-2 * a))
    np.testing.assert_allclose(out2[0, 0], [s2, 1 - s2, 0, 0], rtol=1e-13)


def test_scores_sum_to_rows_times_group():
    # every softmax row of Eq. 4 sums to one
    rng = np.random.default_rng(3)
    hq, hkv, c, n, d = 8, 2, 37, 29, 16
    q = _rand_bf16(rng, (n, hq, d))
    k_all = _rand_bf16(rng, (hkv, c + n, d))
    v_all = _rand_bf16(rng, (hkv, c + n, d))
    _, scores = O.attend_chunk(q, k_all, v_all, c)
    np.testing.assert_allclose(scores.sum(axis=1), n * (hq // hkv), rtol=1e-12)
    assert np.all(scores >= 0)


def test_gqa_identical_heads_scale_scores():
    rng = np.random.default_rng(4)
    c, n, d, g = 11, 9, 8, 3
    q1 = _rand_bf16(rng, (n, 1, d))
    k_all = _rand_bf16(rng, (1, c + n, d))
    v_all = _rand_bf16(rng, (1, c + n, d))
    out1, s1 = O.attend_chunk(q1, k_all, v_all, c)
    outg, sg = O.attend_chunk(np.repeat(q1, g, axis=1), k_all, v_all, c)
    np.testing.assert_allclose(sg, g * s1, rtol=1e-13)
    for h in range(g):
        np.testing.assert_allclose(outg[:, h], out1[:, 0], rtol=1e-13)


def test_gqa_head_to_kv_head_mapping():
    # query heads [g*hk, g*(hk+1)) read KV head hk: make KV head 1's values distinct
    rng = np.random.default_rng(5)
    n, d = 4, 4
    q = _rand_bf16(rng, (n, 4, d))
    k_all = _rand_bf16(rng, (2, n, d))
    v_all = np.stack([np.zeros((n, d)), np.ones((n, d))])
    out, _ = O.attend_chunk(q, k_all, v_all, 0)
    assert np.allclose(out[:, 0:2], 0.0) and np.allclose(out[:, 2:4], 1.0)


def test_cache_slot_permutation_invariance():
    rng = np.random.default_rng(6)
    hq, hkv, c, n, d = 4, 2, 13, 7, 8
    q = _rand_bf16(rng, (n, hq, d))
    k_all = _rand_bf16(rng, (hkv, c + n, d))
    v_all = _rand_bf16(rng, (hkv, c + n, d))
    out, scores = O.attend_chunk(q, k_all, v_all, c)
    perm = rng.permutation(c)
    full = np.concatenate([perm, np.arange(c, c + n)])
    out_p, scores_p = O.attend_chunk(q, k_all[:, full], v_all[:, full], c)
    np.testing.assert_allclose(out_p, out, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(scores_p, scores[:, full], rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- full cache == library attention
def _sdpa_full(q, k, v):
    """Causal attention over the whole prefix in one shot with torch's CPU
    scaled_dot_product_attention (float64), GQA by repeating KV heads."""
    g = q.shape[1] // k.shape[1]
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, g, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, g, axis=1)).permute(1, 0, 2)[None]
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    return o[0].permute(1, 0, 2).numpy()


@pytest.mark.parametrize("chunk", [64, 96, 608])
def test_budget_at_least_prefix_is_full_attention(chunk):
    # Alg. 1 line 8 never fires when M >= N: the "Full Cache" rows of Tab. 1.
    # The result must not depend on the block size either (Tab. 3a's block vs bulk).
    wl = get_workload("tiny")
    qb, kb, vb = layer_inputs(wl, 0)
    q, k, v = (bf16_bits_to_f32(x).astype(np.float64) for x in (qb, kb, vb))
    cache, recs = O.prefill_layer(q, k, v, chunk, budget=wl.n_tokens, segments=wl.segments, merge=True)
    out = np.concatenate([r["out"] for r in recs], axis=0)
    want = _sdpa_full(q, k, v)
    np.testing.assert_allclose(out, want, rtol=1e-9, atol=1e-11)
    assert cache.count == wl.n_tokens
    assert np.array_equal(cache.idx, np.broadcast_to(np.arange(wl.n_tokens), cache.idx.shape))
    assert np.all(cache.w == 1)
    assert np.array_equal(cache.K, k.transpose(1, 0, 2))
    assert np.array_equal(cache.V, v.transpose(1, 0, 2))


# ---------------------------------------------------------------- selection
def test_select_brute_force_and_ties():
    rng = np.random.default_rng(7)
    for trial in range(20):
        m, budget = 50, int(rng.integers(1, 50))
        scores = rng.choice(np.array([0.0, 0.25, 0.5, 1.0, 2.0], dtype=np.float32), size=m)
        tok = rng.permutation(1000)[:m]
        keep = O.select_keep(scores, tok, budget)
        want = sorted(range(m), key=lambda p: (-float(scores[p]), int(tok[p])))[:budget]
        assert sorted(np.nonzero(keep)[0].tolist()) == sorted(want)
        assert keep.sum() == budget
    # all scores equal: the lowest token indices stay
    tok = np.array([9, 3, 7, 1, 5])
    keep = O.select_keep(np.zeros(5, dtype=np.float32), tok, 2)
    assert set(tok[keep].tolist()) == {1, 3}
    # nothing to evict at or below the budget (strict ">" of Alg. 1 line 8)
    assert O.select_keep(np.zeros(5, dtype=np.float32), tok, 5).all()
    assert O.select_keep(np.zeros(5, dtype=np.float32), tok, 9).all()


def test_cache_never_exceeds_budget_and_evicts_exact_excess():
    # Alg. 1 lines 8-11 on the tiny workload with an odd block and budget
    wl = get_workload("tiny")
    qb, kb, vb = layer_inputs(wl, 0)
    q, k, v = (bf16_bits_to_f32(x).astype(np.float64) for x in (qb, kb, vb))
    for merge in (False, True):
        cache = O.LayerCache(wl.n_kv_heads, wl.head_dim, 100, wl.segments, merge)
        seen = 0
        for t0, n in chunk_ranges(wl.n_tokens, 48):
            c = cache.count
            rec = cache.step(t0, q[t0:t0 + n], k[t0:t0 + n], v[t0:t0 + n])
            seen += n
            assert cache.count == min(100, c + n)
            assert (~rec["keep"]).sum(axis=1).tolist() == [max(0, c + n - 100)] * wl.n_kv_heads
            for hk in range(wl.n_kv_heads):
                assert len(set(cache.idx[hk].tolist())) == cache.count       # no token twice
                assert cache.idx[hk].max() < seen
                # multiplicity is conserved: kept + dropped = tokens seen
                assert cache.w[hk].sum() + cache.dropped_w[hk] == seen
            if not merge:
                assert np.all(cache.w == 1)
        # determinism
        cache2, _ = O.prefill_layer(q, k, v, 48, 100, wl.segments, merge)
        assert np.array_equal(cache2.idx, cache.idx) and np.array_equal(cache2.K, cache.K)


def test_slot_rule_kept_rows_stay_new_rows_fill_free_slots():
    hkv, d, budget = 1, 2, 4
    cache = O.LayerCache(hkv, d, budget)
    k0 = np.arange(8, dtype=np.float64).reshape(4, 1, 2)
    cache.compact(0, k0, k0, np.zeros((1, 4), dtype=np.float32))
    assert cache.idx.tolist() == [[0, 1, 2, 3]]
    # candidates: slots 0..3 (tokens 0..3) then tokens 4, 5, 6; keep tokens 1, 3 and 4, 6
    k1 = 100 + np.arange(6, dtype=np.float64).reshape(3, 1, 2)
    scores = np.array([[0, 5, 0, 5, 5, 0.5, 5]], dtype=np.float32)
    rec = cache.compact(4, k1, k1, scores)
    assert rec["keep"].tolist() == [[False, True, False, True, True, False, True]]
    # slots 0 and 2 were freed; token 4 takes slot 0 and token 6 takes slot 2
    assert cache.idx.tolist() == [[4, 1, 6, 3]]
    assert cache.K[0].tolist() == [[100, 101], [2, 3], [104, 105], [6, 7]]
    # partly filled cache going over budget: unused slots count as free, in order
    cache = O.LayerCache(1, 2, 4)
    cache.compact(0, k0[:3], k0[:3], np.zeros((1, 3), dtype=np.float32))
    rec = cache.compact(3, k1, k1, np.array([[1, 0, 1, 0, 1, 1]], dtype=np.float32))
    assert cache.idx.tolist() == [[0, 4, 2, 5]]


# ---------------------------------------------------------------- grid structure and merge (build-defined)
def _load_golden(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


def test_grid_neighbours_hand_worked():
    g = _load_golden("grid_neighbours.json")
    for case in g["cases"]:
        segs = [Segment(*s) for s in case["segments"]]
        for t, want in case["neighbours"].items():
            assert sorted(O.grid_neighbours(int(t), segs)) == sorted(want), (case["name"], t)


def test_grid_neighbours_symmetry_and_degree():
    for wl in WORKLOADS[:4]:
        segs = wl.segments
        vis = segs[0]
        per = vis.grid_h * vis.grid_w
        rng = np.random.default_rng(0)
        for t in rng.integers(0, vis.n_tokens, 200):
            nb = O.grid_neighbours(int(t), segs)
            assert len(nb) == len(set(nb))
            for u in nb:
                assert t in O.grid_neighbours(int(u), segs)                # symmetric
                if not vis.temporal:
                    assert u // per == t // per                               # never across tiles
        # an interior cell has 4 neighbours in a tile, 6 in the middle of a video
        t_int = (vis.n_planes // 2) * per + vis.grid_w + 1
        assert len(O.grid_neighbours(t_int, segs)) == (6 if vis.temporal and vis.n_planes > 2 else 4)
        assert O.grid_neighbours(vis.n_tokens, segs) == []                    # text token


def test_merge_plan_hand_worked():
    g = _load_golden("merge_plan.json")
    for case in g["cases"]:
        segs = [Segment(*s) for s in case["segments"]]
        tok = np.array(case["tok"])
        scores = np.array(case["scores"], dtype=np.float32)
        keep = np.array(case["keep"], dtype=bool)
        dst = O.merge_plan(scores, tok, keep, segs)
        assert dst.tolist() == case["dst"], case["name"]


def test_merge_rows_closed_forms():
    # weights 1 and 1: plain average; then the destination carries weight 2 and a
    # third token of weight 1 gives the 3-token mean: (2*avg + x)/3
    rows = np.array([[1.0, 2.0], [3.0, 6.0], [8.0, 1.0]])
    w = np.array([1, 1, 1])
    r1, w1 = O.merge_rows(w, rows, np.array([-1, 0, -1]))
    assert r1[0].tolist() == [2.0, 4.0] and w1.tolist() == [2, 1, 1]
    assert r1[1].tolist() == [3.0, 6.0]                  # sources are left alone
    r2, w2 = O.merge_rows(w1, r1, np.array([-1, -1, 0]))
    assert r2[0].tolist() == [4.0, 3.0] and w2[0] == 3   # (2*2+8)/3, (2*4+1)/3
    # two sources at once, and the single bf16 rounding: (1 + 1 + 1.0078125)/3 = 1.00260..
    # which rounds to 1.0 (bf16 spacing above 1 is 2^-7)
    rows = np.array([[1.0], [1.0], [1.0078125]])
    r3, w3 = O.merge_rows(np.array([1, 1, 1]), rows, np.array([-1, 0, 0]))
    assert r3[0, 0] == 1.0 and w3[0] == 3
    # merging an identical row changes nothing but the weight
    rows = np.array([[0.33203125, -7.5], [0.33203125, -7.5]])
    r4, w4 = O.merge_rows(np.array([5, 2]), rows, np.array([-1, 0]))
    assert np.array_equal(r4, rows) and w4.tolist() == [7, 2]


def test_merge_conserves_weighted_sum_and_constant_field():
    wl = get_workload("tiny")
    rng = np.random.default_rng(11)
    qb, kb, vb = layer_inputs(wl, 0)
    q, k, v = (bf16_bits_to_f32(x).astype(np.float64) for x in (qb, kb, vb))
    # constant visual field: every merged row must stay equal to that constant
    nvis = wl.segments[0].n_tokens
    kc, vc = k.copy(), v.copy()
    kc[:nvis] = kc[0]
    vc[:nvis] = vc[0]
    cache, recs = O.prefill_layer(q, kc, vc, wl.chunk, wl.budget, wl.segments, merge=True)
    merged_any = False
    for hk in range(wl.n_kv_heads):
        vis = cache.idx[hk] < nvis
        assert np.array_equal(cache.K[hk][vis], np.broadcast_to(kc[0, hk], cache.K[hk][vis].shape))
        assert np.array_equal(cache.V[hk][vis], np.broadcast_to(vc[0, hk], cache.V[hk][vis].shape))
        merged_any |= bool((cache.w[hk] > 1).any())
        assert np.all(cache.w[hk][~vis] == 1)            # text never receives a merge
    assert merged_any
    # one compaction, general field: sum_w(K) over kept+merged sources is preserved up to rounding
    cache = O.LayerCache(wl.n_kv_heads, wl.head_dim, wl.budget, wl.segments, merge=True)
    for t0, n in chunk_ranges(wl.n_tokens, wl.chunk)[:3]:
        tok, w, k_all, _ = cache.candidates(t0, k[t0:t0 + n], v[t0:t0 + n])
        rec = cache.step(t0, q[t0:t0 + n], k[t0:t0 + n], v[t0:t0 + n])
    keep, dst = rec["keep"], rec["dst"]
    for hk in range(wl.n_kv_heads):
        involved = keep[hk] | (dst[hk] >= 0)
        before = (w[hk][involved, None] * k_all[hk][involved]).sum(axis=0)
        after = (cache.w[hk][:, None] * cache.K[hk]).sum(axis=0)
        tol = 2.0 ** -8 * (cache.w[hk][:, None] * np.abs(cache.K[hk])).sum(axis=0)
        assert np.all(np.abs(before - after) <= tol)
        # sources never are destinations and vice versa; destinations are kept visual tokens
        d = dst[hk][dst[hk] >= 0]
        assert keep[hk][d].all() and not keep[hk][dst[hk] >= 0].any()
        assert np.all(tok[hk][d] < nvis) and np.all(tok[hk][dst[hk] >= 0] < nvis)


def test_merge_does_not_change_first_selection():
    wl = get_workload("tiny")
    qb, kb, vb = layer_inputs(wl, 0)
    q, k, v = (bf16_bits_to_f32(x).astype(np.float64) for x in (qb, kb, vb))
    ranges = chunk_ranges(wl.n_tokens, wl.chunk)[:3]           # third block is the first to evict
    kept = []
    for merge in (False, True):
        cache = O.LayerCache(wl.n_kv_heads, wl.head_dim, wl.budget, wl.segments, merge)
        for t0, n in ranges:
            rec = cache.step(t0, q[t0:t0 + n], k[t0:t0 + n], v[t0:t0 + n])
        kept.append(np.sort(cache.idx, axis=1))
        assert (~rec["keep"]).any()
    assert np.array_equal(kept[0], kept[1])


# ---------------------------------------------------------------- query-agnostic scores
def test_keydiff_scores_closed_forms():
    # two opposite keys plus one along +x: mean is along +x; cosines are +1, -1, +1
    k = np.array([[[2.0, 0.0], [-1.0, 0.0], [5.0, 0.0]]])
    np.testing.assert_allclose(O.keydiff_scores(k)[0], [-1.0, 1.0, -1.0])
    # orthogonal to the mean scores 0: keys (1,1), (1,-1) -> mean (1,0); add (0,3)?
    k = np.array([[[1.0, 1.0], [1.0, -1.0]]])
    np.testing.assert_allclose(O.keydiff_scores(k)[0], [-math.sqrt(0.5)] * 2)
    # brute force
    rng = np.random.default_rng(2)
    k = rng.standard_normal((2, 9, 5))
    got = O.keydiff_scores(k)
    for h in range(2):
        mu = [sum(k[h, j, e] for j in range(9)) / 9 for e in range(5)]
        for j in range(9):
            dot = sum(k[h, j, e] * mu[e] for e in range(5))
            nk = math.sqrt(sum(k[h, j, e] ** 2 for e in range(5)))
            nm = math.sqrt(sum(m * m for m in mu))
            assert abs(got[h, j] + dot / (nk * nm)) < 1e-12


# ----------------------------------------------------------------------------
# proxy-query scores (Sec. 3.2, Eq. 4 without a causal mask)
# ----------------------------------------------------------------------------
def test_proxy_scores_against_library_softmax_and_loops():
    from scipy.special import softmax
    rng = np.random.default_rng(21)
    n_obs, hq, hkv, m, d = 5, 6, 2, 23, 8
    q = _rand_bf16(rng, (n_obs, hq, d))
    k = _rand_bf16(rng, (hkv, m, d))
    got = O.proxy_scores(q, k)
    # a library softmax, one head at a time
    want = np.zeros((hkv, m))
    for h in range(hq):
        want[h // (hq // hkv)] += softmax((q[:, h, :] @ k[h // (hq // hkv)].T) / math.sqrt(d), axis=1).sum(axis=0)
    np.testing.assert_allclose(got, want, rtol=1e-12)
    # plain loops on one query head
    h, hk = 4, 1
    col = [0.0] * m
    for r in range(n_obs):
        logit = [sum(q[r, h, x] * k[hk, j, x] for x in range(d)) / math.sqrt(d) for j in range(m)]
        z = sum(math.exp(v) for v in logit)
        for j in range(m):
            col[j] += math.exp(logit[j]) / z
    solo = O.proxy_scores(q[:, h:h + 1, :], k[hk:hk + 1])
    np.testing.assert_allclose(solo[0], col, rtol=1e-12)


def test_proxy_scores_invariants_and_relation_to_block_scores():
    rng = np.random.default_rng(22)
    n_obs, hq, hkv, c, n, d = 7, 4, 2, 9, 6, 8
    q_obs = _rand_bf16(rng, (n_obs, hq, d))
    k_all = _rand_bf16(rng, (hkv, c + n, d))
    v_all = _rand_bf16(rng, (hkv, c + n, d))
    s = O.proxy_scores(q_obs, k_all)
    # every softmax row sums to one
    np.testing.assert_allclose(s.sum(axis=1), n_obs * (hq // hkv), rtol=1e-12)
    # all keys equal: uniform over all candidates, no causal mask
    ku = np.ones((hkv, c + n, d))
    np.testing.assert_allclose(O.proxy_scores(q_obs, ku), n_obs * (hq // hkv) / (c + n), rtol=1e-12)
    # an explicit scale is honoured: scale 0 is uniform whatever the keys
    np.testing.assert_allclose(O.proxy_scores(q_obs, k_all, scale=0.0), n_obs * (hq // hkv) / (c + n), rtol=1e-12)
    # the last row of a block sees every candidate, as a proxy query does: the block scores of
    # a one-row block equal the proxy scores of that row over cache + that row's key
    q1 = _rand_bf16(rng, (1, hq, d))
    _, block_scores = O.attend_chunk(q1, k_all[:, :c + 1], v_all[:, :c + 1], c)
    np.testing.assert_allclose(O.proxy_scores(q1, k_all[:, :c + 1]), block_scores, rtol=1e-12)
    # permuting the candidates permutes the scores
    perm = rng.permutation(c + n)
    np.testing.assert_allclose(O.proxy_scores(q_obs, k_all[:, perm]), s[:, perm], rtol=1e-12)


def test_keydiff_scores_against_loops_and_invariants():
    rng = np.random.default_rng(31)
    hkv, m, d = 2, 17, 6
    k = _rand_bf16(rng, (hkv, m, d))
    got = O.keydiff_scores(k)
    for hk in range(hkv):
        mu = [sum(k[hk, j, x] for j in range(m)) / m for x in range(d)]
        nmu = math.sqrt(sum(v * v for v in mu))
        for j in range(m):
            dot = sum(k[hk, j, x] * mu[x] for x in range(d))
            nk = math.sqrt(sum(k[hk, j, x] ** 2 for x in range(d)))
            assert abs(got[hk, j] + dot / (nk * nmu)) < 1e-12
    assert (np.abs(got) <= 1 + 1e-12).all()                      # a cosine
    np.testing.assert_allclose(O.keydiff_scores(3.5 * k), got, rtol=1e-12)      # scale-free
    perm = rng.permutation(m)
    np.testing.assert_allclose(O.keydiff_scores(k[:, perm]), got[:, perm], rtol=1e-12)
    # the key that is the anchor's own direction scores lowest, its opposite highest
    base = np.zeros((1, 5, 3)); base[0, :, 0] = [1, 2, 3, 4, -0.5]
    s = O.keydiff_scores(base)[0]
    assert np.allclose(s[:4], -1) and np.isclose(s[4], 1)


# ----------------------------------------------------------------------------
# one generation step (Eq. 1 with one query row)
# ----------------------------------------------------------------------------
def test_decode_step_against_library_softmax_loops_and_the_block_routine():
    rng = np.random.default_rng(77)
    hq, hkv, d, m = 6, 2, 8, 19
    g = hq // hkv
    q = rng.standard_normal((hq, d))
    k = rng.standard_normal((hkv, m, d))
    v = rng.standard_normal((hkv, m, d))
    from scipy.special import softmax
    got = O.decode_step(q, k, v)
    # library softmax, one head at a time
    for h in range(hq):
        hk = h // g
        w = softmax(k[hk] @ q[h] / np.sqrt(d))
        np.testing.assert_allclose(got[h], w @ v[hk], rtol=1e-12, atol=1e-14)
    # scalar loops from the definition
    for h in (0, 3, 5):
        hk = h // g
        logit = [sum(q[h, x] * k[hk, j, x] for x in range(d)) / math.sqrt(d) for j in range(m)]
        z = sum(math.exp(t) for t in logit)
        for x in (0, d - 1):
            want = sum(math.exp(logit[j]) / z * v[hk, j, x] for j in range(m))
            assert abs(got[h, x] - want) < 1e-12
    # a one-row block over a cache of m - 1 entries is the same computation
    out_block, _ = O.attend_chunk(q[None], k, v, m - 1)
    np.testing.assert_allclose(got, out_block[0], rtol=1e-12, atol=1e-14)
    # the last row of a longer block sees everything as well
    n = 5
    qb = rng.standard_normal((n, hq, d))
    qb[-1] = q
    out_block, _ = O.attend_chunk(qb, k, v, m - n)
    np.testing.assert_allclose(got, out_block[-1], rtol=1e-12, atol=1e-14)


def test_decode_step_invariants():
    rng = np.random.default_rng(78)
    hq, hkv, d, m = 4, 2, 16, 33
    q = rng.standard_normal((hq, d))
    k = rng.standard_normal((hkv, m, d))
    v = rng.standard_normal((hkv, m, d))
    got = O.decode_step(q, k, v)
    # equal values: the output is that value whatever the weights are
    vc = np.broadcast_to(rng.standard_normal((hkv, 1, d)), v.shape)
    np.testing.assert_allclose(O.decode_step(q, k, vc), np.repeat(vc[:, 0], hq // hkv, axis=0), rtol=1e-12)
    # zero scale: the plain mean of the values
    np.testing.assert_allclose(O.decode_step(q, k, v, scale=0.0), np.repeat(v.mean(axis=1), hq // hkv, axis=0), rtol=1e-12)
    # the order of the keys carries no meaning
    perm = rng.permutation(m)
    np.testing.assert_allclose(O.decode_step(q, k[:, perm], v[:, perm]), got, rtol=1e-12, atol=1e-14)
    # one key: its value
    np.testing.assert_allclose(O.decode_step(q, k[:, :1], v[:, :1]), np.repeat(v[:, 0], hq // hkv, axis=0), rtol=1e-12)
    # a key whose logit dwarfs the rest takes all the weight
    kb = k.copy()
    kb[:, 7] = 0
    qb = np.zeros_like(q); qb[:, 0] = 1.0
    kb[:, :, 0] = -50.0; kb[:, 7, 0] = 50.0
    np.testing.assert_allclose(O.decode_step(qb, kb, v, scale=1.0), np.repeat(v[:, 7], hq // hkv, axis=0), rtol=1e-12, atol=1e-12)
    # convexity: every output channel lies between the extremes of that channel's values
    for h in range(hq):
        hk = h // (hq // hkv)
        assert np.all(got[h] <= v[hk].max(axis=0) + 1e-12) and np.all(got[h] >= v[hk].min(axis=0) - 1e-12)
