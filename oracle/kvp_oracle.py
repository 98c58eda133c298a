"""CPU oracle for block-wise prefill with a fixed-budget KV cache.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the
hot path computes.  It is imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product path, and it shares no code
with the HIP kernels.  All floating-point work is float64 on the
bfloat16-valued inputs; the one place a decision hangs on floating point (which
keys are kept) is taken on the float32 rounding of the scores, the precision
the GPU path stores them in.

What follows the paper, and where:
  * ``attend_chunk``      Eq. 1 (Sec. 2.1) for a block attending over
                          cache U block, and Eq. 4 (Sec. 3.2) for the scores.
  * ``select_keep``       "tokens with lower importance scores are evicted
                          until the cache satisfies the budget M" (Sec. 3.2),
                          Alg. 1 lines 8-11.
  * ``prefill_layer`` / ``LayerCache.step``   the loop of Alg. 1.
  * ``kv_cache_bytes``    Eq. 2 (Sec. 2.2).
  * ``proxy_scores``      Eq. 4 with the proxy queries of Sec. 3.2 (every
                          candidate visible to every proxy query).
  * ``keydiff_scores``    the query-agnostic strategy of Sec. 3.2.
  * ``decode_step``       Eq. 1 (Sec. 2.1) for the one query row of a
                          generation step over cache U generated tokens.

Readings where the paper is silent (each is a choice of this build):
  * the observation queries of Eq. 4 are the block's own queries; their
    softmax rows are summed over rows and over the query heads that share a KV
    head (grouped-query attention); no pooling, no score memory across blocks,
    no protected tokens, no normalisation for causal visibility;
  * selection is independent per KV head; ties keep the lower token index;
  * eviction fires only when ``|C| > M`` and removes exactly ``|C| - M``;
  * softmax scale ``1/sqrt(d_k)``; causal inside the block, cache fully visible.

The grid-neighbour merge (``merge_plan``, ``merge_rows``) is NOT in the paper,
which is eviction-only (App. A); it is defined by this build and is switched
off with ``merge=False``, which is the paper's method.  Its rules:
  M1 a visual token's coordinates (plane, y, x) come from its segment, tokens
     row-major inside a plane;
  M2 neighbours: the 4-connected cells of the same plane, plus the same cell
     of the previous and next plane when the segment is temporal;
  M3 an evicted visual token may merge only into a neighbour that is a
     candidate of the same head at this compaction and is kept;
  M4 it picks the eligible neighbour with the highest score, ties to the
     lower token index; with none eligible it is dropped; one hop only;
  M5 destination rows become weight-averaged K and V from pre-compaction
     values, one round-to-nearest-even to bfloat16; weights are integer
     multiplicities starting at 1;
  M6 weights never bias the logits.

Pins: tests/test_oracle_pins.py checks every function here against closed
forms, brute force, a library attention routine and hand-worked grids.  The
paper prints no worked example or intermediate value for this path, so against
the paper's own numbers parity is unpinned; it is pinned by the definitions and
invariants listed in that test file.
"""
from __future__ import annotations

import numpy as np

TEXT = 0
VISUAL = 1


# ----------------------------------------------------------------------------
# bfloat16 <-> float64
# ----------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 value (ties to even) of float64 ``x``, as float64.
    One rounding, straight from float64.  Domain: zero or bfloat16-normal
    magnitudes, which is all the path produces."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    a = np.abs(x)
    ok = (a == 0) | ((a >= 2.0 ** -126) & (a < 2.0 ** 127))
    if not np.all(ok):
        raise ValueError("round_to_bf16: value outside the normal bfloat16 range")
    u = x.view(np.uint64)
    drop = np.uint64(52 - 7)
    lsb = (u >> drop) & np.uint64(1)
    bias = lsb + ((np.uint64(1) << (drop - np.uint64(1))) - np.uint64(1))
    r = (u + bias) & ~((np.uint64(1) << drop) - np.uint64(1))
    return r.view(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Bit patterns of values that are already bfloat16-representable."""
    f = np.ascontiguousarray(x, dtype=np.float64).astype(np.float32)
    if not np.array_equal(f.astype(np.float64), x):
        raise ValueError("value is not representable in float32")
    u = f.view(np.uint32)
    if np.any(u & np.uint32(0xFFFF)):
        raise ValueError("value is not representable in bfloat16")
    return (u >> np.uint32(16)).astype(np.uint16)


# ----------------------------------------------------------------------------
# Eq. 2
# ----------------------------------------------------------------------------
def kv_cache_bytes(n_layers: int, n_kv_heads: int, head_dim: int, precision_bytes: int, seq_len: int) -> int:
    """Eq. 2: 2 x layers x heads x dim_head x precision x sequence length."""
    return 2 * n_layers * n_kv_heads * head_dim * precision_bytes * seq_len


# ----------------------------------------------------------------------------
# Eq. 1 and Eq. 4 for one block
# ----------------------------------------------------------------------------
def attend_chunk(q, k_all, v_all, c, scale=None):
    """One block of queries over cache U block (Eq. 1), and the importance of
    every key (Eq. 4 summed over the observation queries).

    q      [n, Hq, d]       the block's queries
    k_all  [Hkv, c + n, d]  cached keys (first ``c`` rows) then the block's keys
    v_all  [Hkv, c + n, d]  likewise for values
    Block row r sees every cached key and block keys 0..r.

    Returns ``out [n, Hq, d]`` and ``scores [Hkv, c + n]``, both float64.
    """
    q = np.asarray(q, dtype=np.float64)
    k_all = np.asarray(k_all, dtype=np.float64)
    v_all = np.asarray(v_all, dtype=np.float64)
    n, hq, d = q.shape
    hkv, tot, _ = k_all.shape
    assert tot == c + n and hq % hkv == 0
    g = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((n, hq, d), dtype=np.float64)
    scores = np.zeros((hkv, tot), dtype=np.float64)
    rows = np.arange(n)[:, None]
    cols = np.arange(n)[None, :]
    hidden = cols > rows                      # block key j is hidden from row r when j > r
    for h in range(hq):
        hk = h // g
        s = scale * (q[:, h, :] @ k_all[hk].T)            # [n, c + n]
        s[:, c:][hidden] = -np.inf
        s -= s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v_all[hk]
        scores[hk] += p.sum(axis=0)
    return out, scores


def proxy_scores(q_obs, k_all, scale=None):
    """Importance of every candidate key under proxy queries (Sec. 3.2 as the
    paper words it: the observation queries come from the textual prompt, and
    Eq. 4 is their attention over the keys).  The prompt follows the visual
    tokens, so a proxy query sees every candidate: no causal mask.

    q_obs  [n_obs, Hq, d]
    k_all  [Hkv, m, d]   the candidates of each KV head (cache rows, then block rows)

    Returns ``scores [Hkv, m]``: softmax rows of Eq. 4 summed over the proxy
    queries and over the query heads that share a KV head.
    """
    q_obs = np.asarray(q_obs, dtype=np.float64)
    k_all = np.asarray(k_all, dtype=np.float64)
    n_obs, hq, d = q_obs.shape
    hkv, m, _ = k_all.shape
    assert hq % hkv == 0
    g = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    scores = np.zeros((hkv, m), dtype=np.float64)
    for h in range(hq):
        hk = h // g
        s = scale * (q_obs[:, h, :] @ k_all[hk].T)        # [n_obs, m]
        s -= s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=1, keepdims=True)
        scores[hk] += p.sum(axis=0)
    return scores


# ----------------------------------------------------------------------------
# Eq. 1 for one generation step
# ----------------------------------------------------------------------------
def decode_step(q, k_all, v_all, scale=None):
    """Eq. 1 with one query row per head (Sec. 2.1: during generation only the
    current token's query is new, the keys and values of all earlier tokens are
    reused).  The current token sees every key it is given.

    q      [Hq, d]
    k_all  [Hkv, m, d]   cached keys, then the keys of the generated tokens, the current one last
    v_all  [Hkv, m, d]

    Returns ``out [Hq, d]`` float64.
    """
    q = np.asarray(q, dtype=np.float64)
    k_all = np.asarray(k_all, dtype=np.float64)
    v_all = np.asarray(v_all, dtype=np.float64)
    hq, d = q.shape
    hkv = k_all.shape[0]
    assert hq % hkv == 0
    g = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((hq, d), dtype=np.float64)
    for h in range(hq):
        hk = h // g
        s = scale * (k_all[hk] @ q[h])                    # [m]
        p = np.exp(s - s.max())
        p /= p.sum()
        out[h] = p @ v_all[hk]
    return out


# ----------------------------------------------------------------------------
# Sec. 3.2, query-agnostic scores
# ----------------------------------------------------------------------------
def keydiff_scores(k_all):
    """Query-agnostic importance (Sec. 3.2): the anchor is the mean of the
    candidate keys; a key matters more the less similar it is to the anchor.
    Similarity is the cosine; the score is its negative, so that "keep the
    highest scores" keeps the keys that deviate most.  k_all [Hkv, m, d]."""
    k_all = np.asarray(k_all, dtype=np.float64)
    mu = k_all.mean(axis=1, keepdims=True)
    num = (k_all * mu).sum(axis=2)
    den = np.linalg.norm(k_all, axis=2) * np.linalg.norm(mu, axis=2)
    return -(num / den)


# ----------------------------------------------------------------------------
# selection (Alg. 1 lines 8-11)
# ----------------------------------------------------------------------------
def select_keep(scores32, tok, budget):
    """Mask of the ``budget`` candidates kept: highest score first, equal
    scores by lower token index.  ``scores32`` float32, ``tok`` distinct ints."""
    scores32 = np.asarray(scores32)
    assert scores32.dtype == np.float32
    tok = np.asarray(tok, dtype=np.int64)
    m = len(tok)
    keep = np.zeros(m, dtype=bool)
    if m <= budget:
        keep[:] = True
        return keep
    order = np.lexsort((tok, -scores32.astype(np.float64)))   # primary: score desc; then token asc
    keep[order[:budget]] = True
    return keep


# ----------------------------------------------------------------------------
# grid structure (M1, M2)
# ----------------------------------------------------------------------------
def grid_coords(t, segments):
    """(segment number, plane, y, x) of visual token ``t``; None for text."""
    for si, s in enumerate(segments):
        if s.token_begin <= t < s.token_begin + s.n_tokens:
            if s.kind != VISUAL:
                return None
            u = t - s.token_begin
            per = s.grid_h * s.grid_w
            return si, u // per, (u % per) // s.grid_w, u % s.grid_w
    raise ValueError(f"token {t} outside the prefix")


def grid_neighbours(t, segments):
    """Token indices of the grid neighbours of visual token ``t`` (M2)."""
    co = grid_coords(t, segments)
    if co is None:
        return []
    si, plane, y, x = co
    s = segments[si]
    per = s.grid_h * s.grid_w

    def tok(pl, yy, xx):
        return s.token_begin + pl * per + yy * s.grid_w + xx

    out = []
    if x > 0:
        out.append(tok(plane, y, x - 1))
    if x + 1 < s.grid_w:
        out.append(tok(plane, y, x + 1))
    if y > 0:
        out.append(tok(plane, y - 1, x))
    if y + 1 < s.grid_h:
        out.append(tok(plane, y + 1, x))
    if s.temporal:
        if plane > 0:
            out.append(tok(plane - 1, y, x))
        if plane + 1 < s.n_planes:
            out.append(tok(plane + 1, y, x))
    return out


def merge_plan(scores32, tok, keep, segments):
    """Destination of every candidate (M3, M4): ``dst[p]`` is the candidate
    position that evicted visual candidate ``p`` merges into, or -1."""
    tok = np.asarray(tok, dtype=np.int64)
    m = len(tok)
    pos_of = {int(t): p for p, t in enumerate(tok)}
    dst = np.full(m, -1, dtype=np.int64)
    for p in range(m):
        if keep[p]:
            continue
        best = None
        for nb in grid_neighbours(int(tok[p]), segments):
            r = pos_of.get(nb)
            if r is None or not keep[r]:
                continue
            cand = (-float(scores32[r]), int(tok[r]), r)
            if best is None or cand < best:
                best = cand
        if best is not None:
            dst[p] = best[2]
    return dst


def merge_rows(w, rows, dst):
    """M5 for one tensor: ``rows [m, d]`` pre-compaction candidate rows,
    ``w [m]`` integer multiplicities.  Returns merged rows (only destinations
    change) and new weights."""
    w = np.asarray(w, dtype=np.int64)
    rows = np.asarray(rows, dtype=np.float64)
    new_rows = rows.copy()
    new_w = w.copy()
    for d_pos in np.unique(dst[dst >= 0]):
        srcs = np.nonzero(dst == d_pos)[0]
        total = int(w[d_pos]) + int(w[srcs].sum())
        acc = float(w[d_pos]) * rows[d_pos]
        for s in srcs:
            acc = acc + float(w[s]) * rows[s]
        new_rows[d_pos] = round_to_bf16(acc / total)
        new_w[d_pos] = total
    return new_rows, new_w


# ----------------------------------------------------------------------------
# the cache of one layer, and Alg. 1
# ----------------------------------------------------------------------------
class LayerCache:
    """KV cache of one layer: per KV head, ``count`` slots of
    (token index, multiplicity, K row, V row); ``count <= budget`` always."""

    def __init__(self, n_kv_heads, head_dim, budget, segments=(), merge=False):
        self.hkv, self.d, self.budget = n_kv_heads, head_dim, budget
        self.segments = tuple(segments)
        self.merge = bool(merge)
        self.count = 0
        self.idx = np.zeros((n_kv_heads, 0), dtype=np.int64)
        self.w = np.zeros((n_kv_heads, 0), dtype=np.int64)
        self.K = np.zeros((n_kv_heads, 0, head_dim), dtype=np.float64)
        self.V = np.zeros((n_kv_heads, 0, head_dim), dtype=np.float64)
        self.dropped_w = np.zeros(n_kv_heads, dtype=np.int64)   # multiplicity lost to plain eviction

    def candidates(self, t0, k, v):
        """Cache rows followed by the block's rows (Alg. 1 line 7)."""
        k = np.asarray(k, dtype=np.float64)
        v = np.asarray(v, dtype=np.float64)
        n = k.shape[0]
        tok = np.concatenate([self.idx, np.broadcast_to(np.arange(t0, t0 + n), (self.hkv, n))], axis=1)
        w = np.concatenate([self.w, np.ones((self.hkv, n), dtype=np.int64)], axis=1)
        k_all = np.concatenate([self.K, k.transpose(1, 0, 2)], axis=1)
        v_all = np.concatenate([self.V, v.transpose(1, 0, 2)], axis=1)
        return tok, w, k_all, v_all

    def attend(self, t0, q, k, v, scale=None):
        """Eq. 1 / Eq. 4 for the block starting at token ``t0``.
        q [n, Hq, d], k, v [n, Hkv, d].  Does not change the cache."""
        _, _, k_all, v_all = self.candidates(t0, k, v)
        return attend_chunk(q, k_all, v_all, self.count, scale)

    def proxy(self, t0, q_obs, k, v, scale=None):
        """Scores of the candidates of the block starting at ``t0`` under proxy
        queries ``q_obs [n_obs, Hq, d]``.  Does not change the cache."""
        _, _, k_all, _ = self.candidates(t0, k, v)
        return proxy_scores(q_obs, k_all, scale)

    def keydiff(self, t0, k, v):
        """Query-agnostic scores of the candidates of the block starting at
        ``t0``.  Does not change the cache."""
        _, _, k_all, _ = self.candidates(t0, k, v)
        return keydiff_scores(k_all)

    def compact(self, t0, k, v, scores32):
        """Append the block and, if over budget, evict (Alg. 1 lines 7-11),
        merging evicted visual tokens when ``merge`` is on.
        Returns a record of the decisions: per head ``keep`` and ``dst`` over
        the candidate positions, and the candidates' token indices."""
        tok, w, k_all, v_all = self.candidates(t0, k, v)
        c, n, mb = self.count, k.shape[0], self.budget
        tot = c + n
        scores32 = np.asarray(scores32)
        assert scores32.dtype == np.float32 and scores32.shape == (self.hkv, tot)
        keep_all = np.ones((self.hkv, tot), dtype=bool)
        dst_all = np.full((self.hkv, tot), -1, dtype=np.int64)
        if tot <= mb:
            self.idx, self.w, self.K, self.V, self.count = tok, w, k_all, v_all, tot
            return {"tok": tok, "keep": keep_all, "dst": dst_all}
        new_idx = np.empty((self.hkv, mb), dtype=np.int64)
        new_w = np.empty((self.hkv, mb), dtype=np.int64)
        new_k = np.empty((self.hkv, mb, self.d), dtype=np.float64)
        new_v = np.empty((self.hkv, mb, self.d), dtype=np.float64)
        for hk in range(self.hkv):
            keep = select_keep(scores32[hk], tok[hk], mb)
            rows_k, rows_v, wt = k_all[hk], v_all[hk], w[hk]
            if self.merge:
                dst = merge_plan(scores32[hk], tok[hk], keep, self.segments)
                rows_k, wk = merge_rows(w[hk], k_all[hk], dst)
                rows_v, wv = merge_rows(w[hk], v_all[hk], dst)
                assert np.array_equal(wk, wv)
                wt = wk
                dst_all[hk] = dst
                self.dropped_w[hk] += int(w[hk][(~keep) & (dst < 0)].sum())
            else:
                self.dropped_w[hk] += int(w[hk][~keep].sum())
            keep_all[hk] = keep
            # slot rule: kept cache rows stay where they are; kept block rows,
            # in ascending token order, fill the free slots in ascending order
            slot_src = np.full(mb, -1, dtype=np.int64)
            free = []
            for s in range(mb):
                if s < c and keep[s]:
                    slot_src[s] = s
                else:
                    free.append(s)
            new_kept = [p for p in range(c, tot) if keep[p]]
            assert len(new_kept) == len(free)
            for s, p in zip(free, new_kept):
                slot_src[s] = p
            new_idx[hk] = tok[hk][slot_src]
            new_w[hk] = wt[slot_src]
            new_k[hk] = rows_k[slot_src]
            new_v[hk] = rows_v[slot_src]
        self.idx, self.w, self.K, self.V, self.count = new_idx, new_w, new_k, new_v, mb
        return {"tok": tok, "keep": keep_all, "dst": dst_all}

    def step(self, t0, q, k, v, scale=None):
        """One iteration of Alg. 1 for this layer: attend, score, compact."""
        out, scores = self.attend(t0, q, k, v, scale)
        scores32 = scores.astype(np.float32)
        rec = self.compact(t0, k, v, scores32)
        rec.update(out=out, scores=scores, scores32=scores32)
        return rec


def prefill_layer(q, k, v, chunk, budget, segments=(), merge=False, scale=None):
    """Alg. 1 for one layer.  q [N, Hq, d], k, v [N, Hkv, d] float64 (bfloat16
    values).  Returns the final cache and the per-block records."""
    n_tok, hkv, d = k.shape
    cache = LayerCache(hkv, d, budget, segments, merge)
    recs = []
    t0 = 0
    while t0 < n_tok:
        n = min(chunk, n_tok - t0)
        recs.append(cache.step(t0, q[t0:t0 + n], k[t0:t0 + n], v[t0:t0 + n], scale))
        t0 += n
    return cache, recs
