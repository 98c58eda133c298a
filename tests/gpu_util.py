"""Helpers of the GPU parity tests: bf16 plumbing and the lock-step protocol.

Lock-step: before every block the GPU cache of the layer is loaded with the
oracle's cache, so that both sides see identical inputs; `out` and the scores
are compared, then both compact with the ORACLE's float32 scores and the kept
sets, merge destinations, weights and rows are compared slot for slot."""
import numpy as np
import torch

import paper_2604_16734_amd as K
from kvp_workload import bf16_bits_to_f32, chunk_ranges, bits_to_torch, torch_to_bits
from oracle import kvp_oracle as O

OUT_TOL = 2e-2        # max relative error of attention outputs (bf16 in, fp32 accumulate)
SCORE_RTOL = 1e-3     # importance scores
# The only absolute slack: a softmax weight below the smallest normal fp32 number (1.18e-38) may be
# flushed to zero on the GPU while float64 keeps it; a score adds up at most one such weight per
# contributing row.  Everything larger must meet the relative bar.
SCORE_ATOL_PER_ROW = 2e-38


def torch_bf16_to_f64(t):
    return O.bf16_bits_to_f64(torch_to_bits(t))


def f64_to_torch_bf16(x, device="cuda:0"):
    return bits_to_torch(O.f64_to_bf16_bits(x), device)


def out_rel_err(out_gpu_f64, out_ref):
    """Per (row, head): max_c |o - o_ref| / max_c |o_ref|; returns the max."""
    num = np.abs(out_gpu_f64 - out_ref).max(axis=-1)
    den = np.abs(out_ref).max(axis=-1)
    return float((num / den).max())


def check_scores(scores_gpu, scores_ref, n_rows_times_group):
    tol = SCORE_RTOL * np.abs(scores_ref) + SCORE_ATOL_PER_ROW * n_rows_times_group
    bad = np.abs(scores_gpu.astype(np.float64) - scores_ref) > tol
    assert not bad.any(), "scores off at %s: gpu %s ref %s" % (
        np.argwhere(bad)[:5].tolist(), scores_gpu[bad][:5], scores_ref[bad][:5])


def upload_state(cache, layer, oc):
    """Copy the oracle's LayerCache into the GPU cache of `layer`."""
    k, v, idx, w, _, _ = _views(cache, layer)
    c = oc.count
    if c:
        k[:, :c] = f64_to_torch_bf16(oc.K)
        v[:, :c] = f64_to_torch_bf16(oc.V)
        idx[:, :c] = torch.from_numpy(oc.idx.astype(np.int32)).to(idx.device)
        w[:, :c] = torch.from_numpy(oc.w.astype(np.float32)).to(w.device)


def _views(cache, layer):
    return cache.decode_ready(layer)


def compare_state(cache, layer, oc, merged_ulp=1):
    k, v, idx, w, count, _ = _views(cache, layer)
    assert count == oc.count
    c = oc.count
    assert np.array_equal(idx[:, :c].cpu().numpy().astype(np.int64), oc.idx), "token indices differ"
    assert np.array_equal(w[:, :c].cpu().numpy().astype(np.int64), oc.w), "weights differ"
    for name, t, ref in (("K", k, oc.K), ("V", v, oc.V)):
        gb = torch_to_bits(t[:, :c]).astype(np.int64)
        rb = O.f64_to_bf16_bits(ref).astype(np.int64)
        plain = oc.w == 1
        assert np.array_equal(gb[plain], rb[plain]), name + " rows that were never merged differ"
        # merged rows: at most one bf16 ulp (bit patterns of same-sign neighbours differ by 1)
        diff = np.abs(gb[~plain] - rb[~plain])
        assert diff.max(initial=0) <= merged_ulp, "%s merged rows differ by %d ulp" % (name, diff.max())
    return int((oc.w > 1).sum())


def lockstep_layer(wl, layer, cache, qb, kb, vb, merge, chunk=None, budget=None, max_chunks=None,
                   device="cuda:0", stats=None, blocks=None, own_scores=True):
    """Runs one layer of `wl` through GPU and oracle in lock-step; asserts parity.
    `blocks`: explicit (first token, length) pairs instead of fixed-size blocks.

    Every block that evicts is run twice from the oracle's state.  First pass: the library
    compacts on its OWN scores, which are read back and compared with the oracle's (Eq. 4).
    Second pass (the graded one): the state is uploaded again, the block is attended again and
    compacted with the ORACLE's float32 scores; kept sets, merge plans, weights and rows must
    then agree slot for slot."""
    chunk = chunk or wl.chunk
    budget = budget or wl.budget
    q64, k64, v64 = (bf16_bits_to_f32(x).astype(np.float64) for x in (qb, kb, vb))
    qt, kt, vt = (bits_to_torch(x, device) for x in (qb, kb, vb))
    oc = O.LayerCache(wl.n_kv_heads, wl.head_dim, budget, wl.segments, merge)
    g = wl.n_q_heads // wl.n_kv_heads
    worst_out, worst_sc, n_merged, n_scored = 0.0, 0.0, 0, 0
    for ci, (t0, n) in enumerate(blocks if blocks is not None else chunk_ranges(wl.n_tokens, chunk)):
        if max_chunks is not None and ci >= max_chunks:
            break
        c = oc.count
        out_ref, scores_ref = oc.attend(t0, q64[t0:t0 + n], k64[t0:t0 + n], v64[t0:t0 + n])
        if own_scores and c + n > budget:
            upload_state(cache, layer, oc)
            cache.set_state(layer, c, t0)
            cache.prefill_chunk(layer, t0, qt[t0:t0 + n], kt[t0:t0 + n], vt[t0:t0 + n])
            cache.compact(layer)
            own, _, _ = cache.debug_last(layer)
            own = own.cpu().numpy()
            check_scores(own, scores_ref, n * g)
            np.testing.assert_allclose(own.sum(axis=1, dtype=np.float64), n * g, rtol=1e-4)
            nz = scores_ref > 1e-30
            worst_sc = max(worst_sc, float((np.abs(own - scores_ref)[nz] / scores_ref[nz]).max()))
            n_scored += 1
        upload_state(cache, layer, oc)
        cache.set_state(layer, c, t0)
        out = cache.prefill_chunk(layer, t0, qt[t0:t0 + n], kt[t0:t0 + n], vt[t0:t0 + n])
        err = out_rel_err(torch_bf16_to_f64(out), out_ref)
        assert err <= OUT_TOL, "block %d: out rel err %.3g" % (ci, err)
        worst_out = max(worst_out, err)
        scores32 = scores_ref.astype(np.float32)
        ov = torch.from_numpy(scores32).to(device).contiguous()
        cache.compact(layer, ov)
        rec = oc.compact(t0, k64[t0:t0 + n], v64[t0:t0 + n], scores32)
        if c + n > budget:
            used, keep, dst = cache.debug_last(layer)
            assert np.array_equal(used.cpu().numpy(), scores32)
            assert np.array_equal(keep.cpu().numpy().astype(bool), rec["keep"]), "kept sets differ at block %d" % ci
            assert np.array_equal(dst.cpu().numpy().astype(np.int64), rec["dst"]), "merge plan differs at block %d" % ci
        n_merged = max(n_merged, compare_state(cache, layer, oc))
    if stats is not None:
        stats.update(out=worst_out, merged=n_merged, score_rel=worst_sc, scored_blocks=n_scored)
    return oc


def jaccard(a, b):
    a, b = set(int(x) for x in a), set(int(x) for x in b)
    return len(a & b) / max(1, len(a | b))
