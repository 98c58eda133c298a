"""Host-side order of calls for a whole prefill: every block through every layer.

Alg. 1 of the paper is one loop per layer: append the block, attend, score, evict.
The two calls of a layer (kvp_prefill_chunk, then kvp_compact) must stay in
order, but the compaction of a layer has nothing to do with the attention of the
next layer: in a model, what follows a layer's attention is its MLP and the next
layer, and none of that reads the cache being compacted.  `Prefill` therefore can
put every kvp_compact on a second stream, where it runs beside the
kvp_prefill_chunk calls that follow.  The loop over the layers and the events
between the two streams live in the library (kvp_prefill_block): one call per
block, so that the host keeps ahead of the GPU.

Both streams have the default priority.

`Prefill` needs every layer's Q, K, V of a block at once, which a benchmark on
synthetic layers has and a model does not: there, layer l + 1 only exists once
layer l is through.  `LayerwisePrefill` is the order of calls for that case:
one attention call per layer as the block moves up the stack, and one
kvp_compact_layers for the stack when the block is through, which compacts (and,
for proxy or key-only scoring, scores) the layers in groups of up to 16 per
kernel launch.
"""
from __future__ import annotations

from . import binding as B


class Prefill:
    """Drives `cache` over blocks and layers.  `overlap=True` needs a cache with
    scratch_sets >= 2 and uses a second stream for the compactions."""

    def __init__(self, cache, n_layers, overlap=False):
        import torch
        self.torch = torch
        self.cache = cache
        self.n_layers = n_layers
        self.overlap = bool(overlap)
        if self.overlap and (int(cache.cfg.scratch_sets) or 1) < 2:
            raise ValueError("overlap needs a cache created with scratch_sets >= 2")
        self.side = torch.cuda.Stream(device=cache.device) if self.overlap else None

    def _streams(self):
        main = self.torch.cuda.current_stream(self.cache.device).cuda_stream
        return main, (self.side.cuda_stream if self.side is not None else None)

    def block(self, t0, qkv_of_layer, out_of_layer=None, obs_of_layer=None, keydiff=False):
        """One block of the prefix through all layers.  `qkv_of_layer(l)` gives the block's
        (q, k, v) of layer l, `out_of_layer(l)` the tensor the attention output goes to (or None).
        The candidates are scored by the block's own queries, or by the proxy queries
        `obs_of_layer(l)`, or (`keydiff`) by the keys alone.  Returns the list of outputs."""
        cache, torch = self.cache, self.torch
        bf = torch.bfloat16
        qs, ks, vs, outs, obs = [], [], [], [], []
        n = None
        for layer in range(self.n_layers):
            q, k, v = qkv_of_layer(layer)
            n = q.shape[0]
            assert q.shape == (n, cache.cfg.n_q_heads, cache.cfg.head_dim)
            assert k.shape == v.shape == (n, cache.cfg.n_kv_heads, cache.cfg.head_dim)
            out = out_of_layer(layer) if out_of_layer else None
            if out is None:
                out = torch.empty_like(q)
            assert out.shape == q.shape
            qs.append(q); ks.append(k); vs.append(v); outs.append(out)
            if obs_of_layer is not None and not keydiff:
                o = obs_of_layer(layer)
                assert o.shape[1:] == q.shape[1:] and (not obs or o.shape[0] == obs[0].shape[0])
                obs.append(o)
        scoring = B.KVP_SCORE_KEYDIFF if keydiff else (B.KVP_SCORE_PROXY if obs else B.KVP_SCORE_OWN)
        ptr = lambda ts: [cache._ptr(t, bf) for t in ts]
        main, side = self._streams()
        rc = B.kvp_prefill_block(cache.handle, t0, n, ptr(qs), ptr(ks), ptr(vs), ptr(outs), scoring,
                                 ptr(obs) if obs else None, obs[0].shape[0] if obs else 0, main, side)
        B._check(rc, "kvp_prefill_block")
        if self.side is not None:
            # the compactions just enqueued on the side stream read the block's K and V after this
            # call returns: tell torch's allocator, so that memory the caller drops now is not
            # handed out again before the side stream is done with it
            for t in ks + vs:
                t.record_stream(self.side)
        return outs

    def finish(self):
        """Make the current stream wait for the compactions still in flight."""
        main, side = self._streams()
        B._check(B.kvp_prefill_join(self.cache.handle, main, side), "kvp_prefill_join")


class LayerwisePrefill:
    """One block at a time, one layer at a time: `layer(...)` for layers 0, 1, ... as the model
    produces their Q, K, V, then `end_block()`.  The cache must have been created with
    scratch_sets >= n_layers (every layer stays pending until the block is through)."""

    def __init__(self, cache, n_layers):
        if (int(cache.cfg.scratch_sets) or 1) < n_layers:
            raise ValueError("a scratch set per layer is needed: create the cache with scratch_sets >= n_layers")
        self.cache = cache
        self.n_layers = n_layers
        self._held = []          # K, V and proxy queries of the block: read again by end_block()
        self._next = 0
        cache.set_deferred_scoring(1)

    def layer(self, layer, t0, q, k, v, out=None, q_obs=None, keydiff=False):
        """Attention of the block for `layer` (Eq. 1); the scores come from the block's own queries
        in the same launch, or later (end_block) from `q_obs` or from the keys alone."""
        if layer != self._next:
            raise ValueError("layers go in order: expected layer %d" % self._next)
        if keydiff:
            out = self.cache.prefill_chunk_keydiff(layer, t0, q, k, v, out=out)
        elif q_obs is not None:
            out = self.cache.prefill_chunk_proxy(layer, t0, q, k, v, q_obs, out=out)
        else:
            out = self.cache.prefill_chunk(layer, t0, q, k, v, out=out)
        self._held.append((k, v, q_obs))
        self._next += 1
        return out

    def end_block(self):
        """Scores still to come, then select, merge and move, for all layers of the block."""
        if self._next != self.n_layers:
            raise ValueError("the block has only been through %d of %d layers" % (self._next, self.n_layers))
        self.cache.compact_layers(0, self.n_layers)
        self._held.clear()       # enqueued on the same stream: the allocator may hand the memory out again
        self._next = 0
