"""Host-side order of calls for a whole prefill: every block through every layer.

Alg. 1 of the paper is one loop per layer: append the block, attend, score, evict.
The two calls of a layer (kvp_prefill_chunk, then kvp_compact) must stay in
order, but the compaction of a layer has nothing to do with the attention of the
next layer: in a model, what follows a layer's attention is its MLP and the next
layer, and none of that reads the cache being compacted.  `Prefill` therefore can
put every kvp_compact on a second stream, where it runs beside the
kvp_prefill_chunk calls that follow; events keep the two hazards in order:

  * a layer's next block waits for that layer's compaction, and
  * a scratch set (layer mod scratch_sets) waits for the compaction of the last
    layer that used it.

Both streams have the default priority.
"""
from __future__ import annotations


class Prefill:
    """Drives `cache` over blocks and layers.  `overlap=True` needs a cache with
    scratch_sets >= 2 and uses a second stream for the compactions."""

    def __init__(self, cache, n_layers, overlap=False):
        import torch
        self.torch = torch
        self.cache = cache
        self.n_layers = n_layers
        self.overlap = bool(overlap)
        self.n_sets = int(cache.cfg.scratch_sets) or 1
        if self.overlap and self.n_sets < 2:
            raise ValueError("overlap needs a cache created with scratch_sets >= 2")
        if self.overlap:
            dev = cache.device
            self.side = torch.cuda.Stream(device=dev)
            self.compacted = [torch.cuda.Event() for _ in range(n_layers)]
            self.attended = [torch.cuda.Event() for _ in range(n_layers)]
            for e in self.compacted:
                e.record(torch.cuda.current_stream(dev))

    def block(self, t0, qkv_of_layer, out_of_layer=None, obs_of_layer=None, keydiff=False):
        """One block of the prefix through all layers.  `qkv_of_layer(l)` gives the block's
        (q, k, v) of layer l, `out_of_layer(l)` the tensor the attention output goes to (or None).
        The candidates are scored by the block's own queries, or by the proxy queries
        `obs_of_layer(l)`, or (`keydiff`) by the keys alone.  Returns the list of outputs."""
        cache, torch = self.cache, self.torch
        outs = []

        def attend(layer, q, k, v):
            out = out_of_layer(layer) if out_of_layer else None
            if keydiff:
                return cache.prefill_chunk_keydiff(layer, t0, q, k, v, out=out)
            if obs_of_layer is not None:
                return cache.prefill_chunk_proxy(layer, t0, q, k, v, obs_of_layer(layer), out=out)
            return cache.prefill_chunk(layer, t0, q, k, v, out=out)
        if not self.overlap:
            for layer in range(self.n_layers):
                q, k, v = qkv_of_layer(layer)
                outs.append(attend(layer, q, k, v))
                cache.compact(layer)
            return outs
        main = torch.cuda.current_stream(cache.device)
        for layer in range(self.n_layers):
            q, k, v = qkv_of_layer(layer)
            main.wait_event(self.compacted[layer])
            if self.n_layers > self.n_sets:
                main.wait_event(self.compacted[(layer - self.n_sets) % self.n_layers])
            outs.append(attend(layer, q, k, v))
            self.attended[layer].record(main)
            self.side.wait_event(self.attended[layer])
            cache.compact(layer, stream=self.side)
            self.compacted[layer].record(self.side)
        return outs

    def finish(self):
        """Make the current stream wait for the compactions still in flight."""
        if self.overlap:
            self.torch.cuda.current_stream(self.cache.device).wait_stream(self.side)
