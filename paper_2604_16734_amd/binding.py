"""ctypes binding of libkvp.so: the same names and arguments as include/kvp.h.

Device pointers are plain integers (``tensor.data_ptr()``); streams are the
integer handle of a HIP stream (``torch.cuda.current_stream().cuda_stream``).
``Cache`` is a convenience holder that owns the device buffer as a torch tensor
and passes tensors' pointers through; it computes nothing.
"""
import ctypes
import os
import re

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libkvp.so")
_HEADER = os.path.join(os.path.dirname(_HERE), "include", "kvp.h")

KVP_OK, KVP_EINVAL, KVP_ESTATE, KVP_ENOMEM, KVP_EDEVICE = 0, -1, -2, -3, -4
KVP_TEXT, KVP_VISUAL = 0, 1
KVP_FLAG_DRY_RUN = 1
KERNEL_KINDS = ("attention", "colsum", "select", "merge", "move", "rowstat", "keydiff", "decode")


class KvpError(RuntimeError):
    def __init__(self, code, what):
        super().__init__("%s: %s (%d)" % (what, kvp_strerror(code), code))
        self.code = code


class KvpSegment(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("token_begin", "n_tokens", "kind", "grid_h", "grid_w", "n_planes", "temporal")]


class KvpConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "n_q_heads", "n_kv_heads", "head_dim", "budget", "chunk_max",
                 "merge", "scratch_sets", "flags")] + [("softmax_scale", ctypes.c_float)]


class KvpView(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("token_idx", ctypes.c_void_p),
                ("weight", ctypes.c_void_p), ("count", ctypes.c_int32), ("budget", ctypes.c_int32),
                ("next_token", ctypes.c_int32)]


class KvpKernelStat(ctypes.Structure):
    _fields_ = [("launches", ctypes.c_int64), ("layers", ctypes.c_int64), ("total_ms", ctypes.c_double)]


_lib = None


def library_path():
    return _LIB_PATH


def declared_symbols():
    """Names of the functions include/kvp.h declares."""
    text = open(_HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvp_[a-z_]+)\s*\(", text)))


def lib():
    """The loaded library.  Raises if it has not been built: there is no other path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                "libkvp.so is missing at %s; build it with `python -m paper_2604_16734_amd.build`"
                % _LIB_PATH)
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        P = ctypes.POINTER
        L.kvp_strerror.restype = ctypes.c_char_p
        L.kvp_strerror.argtypes = [ctypes.c_int]
        L.kvp_kernel_name.restype = ctypes.c_char_p
        L.kvp_kernel_name.argtypes = [i32]
        L.kvp_cache_bytes.restype = sz
        L.kvp_cache_bytes.argtypes = [P(KvpConfig)]
        L.kvp_persistent_bytes.restype = sz
        L.kvp_persistent_bytes.argtypes = [P(KvpConfig)]
        L.kvp_init_cache.restype = ctypes.c_int
        L.kvp_init_cache.argtypes = [P(KvpConfig), P(KvpSegment), i32, vp, sz, vp, P(vp)]
        L.kvp_prefill_chunk.restype = ctypes.c_int
        L.kvp_prefill_chunk.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp]
        L.kvp_prefill_chunk_proxy.restype = ctypes.c_int
        L.kvp_prefill_chunk_proxy.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, i32, vp]
        L.kvp_prefill_chunk_keydiff.restype = ctypes.c_int
        L.kvp_prefill_chunk_keydiff.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp]
        L.kvp_prefill_block.restype = ctypes.c_int
        L.kvp_prefill_block.argtypes = [vp, i32, i32, P(vp), P(vp), P(vp), P(vp), i32, P(vp), i32, vp, vp]
        L.kvp_prefill_join.restype = ctypes.c_int
        L.kvp_prefill_join.argtypes = [vp, vp, vp]
        L.kvp_compact.restype = ctypes.c_int
        L.kvp_compact.argtypes = [vp, i32, vp, vp]
        L.kvp_set_deferred_scoring.restype = ctypes.c_int
        L.kvp_set_deferred_scoring.argtypes = [vp, i32]
        L.kvp_compact_layers.restype = ctypes.c_int
        L.kvp_compact_layers.argtypes = [vp, i32, i32, vp]
        L.kvp_decode_step.restype = ctypes.c_int
        L.kvp_decode_step.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp]
        L.kvp_decode_step_static.restype = ctypes.c_int
        L.kvp_decode_step_static.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp]
        L.kvp_decode_ready.restype = ctypes.c_int
        L.kvp_decode_ready.argtypes = [vp, i32, P(KvpView)]
        L.kvp_set_state.restype = ctypes.c_int
        L.kvp_set_state.argtypes = [vp, i32, i32, i32]
        L.kvp_set_attention_shape.restype = ctypes.c_int
        L.kvp_set_attention_shape.argtypes = [vp, i32]
        L.kvp_set_score_sweep.restype = ctypes.c_int
        L.kvp_set_score_sweep.argtypes = [vp, i32]
        L.kvp_debug_last.restype = ctypes.c_int
        L.kvp_debug_last.argtypes = [vp, i32, P(vp), P(vp), P(vp), P(i32), P(i32)]
        L.kvp_debug_totals.restype = ctypes.c_int
        L.kvp_debug_totals.argtypes = [vp, P(vp)]
        L.kvp_profile_enable.restype = ctypes.c_int
        L.kvp_profile_enable.argtypes = [vp, i32]
        L.kvp_profile_read.restype = ctypes.c_int
        L.kvp_profile_read.argtypes = [vp, P(KvpKernelStat)]
        L.kvp_probe_mfma.restype = ctypes.c_int
        L.kvp_probe_mfma.argtypes = [vp, sz, i32, i32, vp, P(ctypes.c_double)]
        L.kvp_probe_copy.restype = ctypes.c_int
        L.kvp_probe_copy.argtypes = [vp, vp, sz, i32, vp]
        L.kvp_free_cache.restype = None
        L.kvp_free_cache.argtypes = [vp]
        _lib = L
    return _lib


def _segments(segs):
    arr = (KvpSegment * len(segs))()
    for i, s in enumerate(segs):
        if isinstance(s, KvpSegment):
            arr[i] = s
        else:
            arr[i] = KvpSegment(s.token_begin, s.n_tokens, s.kind, s.grid_h, s.grid_w, s.n_planes, s.temporal)
    return arr


# ---- one function per entry point, same names --------------------------------
def kvp_strerror(code):
    return lib().kvp_strerror(code).decode()


def kvp_kernel_name(kind):
    return lib().kvp_kernel_name(kind).decode()


def kvp_cache_bytes(cfg):
    return lib().kvp_cache_bytes(ctypes.byref(cfg))


def kvp_persistent_bytes(cfg):
    return lib().kvp_persistent_bytes(ctypes.byref(cfg))


def kvp_init_cache(cfg, segs, device_buf, device_bytes, stream=0):
    """Returns (code, handle)."""
    arr = _segments(segs)
    out = ctypes.c_void_p()
    rc = lib().kvp_init_cache(ctypes.byref(cfg), arr, len(segs), device_buf, device_bytes, stream,
                              ctypes.byref(out))
    return rc, out.value


def kvp_prefill_chunk(handle, layer, token_begin, n_tokens, q, k, v, out, stream=0):
    return lib().kvp_prefill_chunk(handle, layer, token_begin, n_tokens, q, k, v, out, stream)


def kvp_prefill_chunk_proxy(handle, layer, token_begin, n_tokens, q, k, v, out, q_obs, n_obs, stream=0):
    return lib().kvp_prefill_chunk_proxy(handle, layer, token_begin, n_tokens, q, k, v, out, q_obs, n_obs, stream)


def kvp_prefill_chunk_keydiff(handle, layer, token_begin, n_tokens, q, k, v, out, stream=0):
    return lib().kvp_prefill_chunk_keydiff(handle, layer, token_begin, n_tokens, q, k, v, out, stream)


def kvp_decode_step(handle, layer, q, k_tail, v_tail, n_tail, out, stream=0):
    return lib().kvp_decode_step(handle, layer, q, k_tail, v_tail, n_tail, out, stream)


def kvp_decode_step_static(handle, layer, q, k_tail, v_tail, n_tail, out, stream=0):
    return lib().kvp_decode_step_static(handle, layer, q, k_tail, v_tail, n_tail, out, stream)


KVP_SCORE_OWN, KVP_SCORE_PROXY, KVP_SCORE_KEYDIFF = 0, 1, 2
KVP_STATIC_SCRATCH_BYTES, KVP_STATIC_MIN_SPLITS = 1 << 20, 16


def _ptr_array(ptrs):
    return (ctypes.c_void_p * len(ptrs))(*ptrs)


def kvp_prefill_block(handle, token_begin, n_tokens, q, k, v, out, scoring=KVP_SCORE_OWN, q_obs=None, n_obs=0,
                      stream=0, side_stream=None):
    """q, k, v, out, q_obs: sequences of n_layers device pointers."""
    obs = _ptr_array(q_obs) if q_obs is not None else None
    return lib().kvp_prefill_block(handle, token_begin, n_tokens, _ptr_array(q), _ptr_array(k), _ptr_array(v),
                                   _ptr_array(out), scoring, obs, n_obs, stream, side_stream)


def kvp_prefill_join(handle, stream=0, side_stream=None):
    return lib().kvp_prefill_join(handle, stream, side_stream)


def kvp_compact(handle, layer, scores_override=None, stream=0):
    return lib().kvp_compact(handle, layer, scores_override, stream)


def kvp_set_deferred_scoring(handle, on):
    return lib().kvp_set_deferred_scoring(handle, on)


def kvp_compact_layers(handle, first_layer, n_layers, stream=0):
    return lib().kvp_compact_layers(handle, first_layer, n_layers, stream)


def kvp_decode_ready(handle, layer):
    """Returns (code, KvpView)."""
    view = KvpView()
    rc = lib().kvp_decode_ready(handle, layer, ctypes.byref(view))
    return rc, view


def kvp_set_state(handle, layer, count, next_token):
    return lib().kvp_set_state(handle, layer, count, next_token)


def kvp_set_attention_shape(handle, shape):
    return lib().kvp_set_attention_shape(handle, shape)


def kvp_set_score_sweep(handle, fused):
    return lib().kvp_set_score_sweep(handle, int(fused))


def kvp_debug_last(handle, layer):
    """Returns (code, scores_ptr, keep_ptr, dst_ptr, n_cand, stride)."""
    s, k, d = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
    n, st = ctypes.c_int32(), ctypes.c_int32()
    rc = lib().kvp_debug_last(handle, layer, ctypes.byref(s), ctypes.byref(k), ctypes.byref(d),
                              ctypes.byref(n), ctypes.byref(st))
    return rc, s.value, k.value, d.value, n.value, st.value


TOTALS = ("evicting_heads", "moved_rows", "merge_destinations", "merge_sources")


def kvp_debug_totals(handle):
    """Returns (code, device pointer to len(TOTALS) uint64 counters)."""
    p = ctypes.c_void_p()
    rc = lib().kvp_debug_totals(handle, ctypes.byref(p))
    return rc, p.value


def kvp_profile_enable(handle, on):
    return lib().kvp_profile_enable(handle, int(on))


def kvp_profile_read(handle):
    """Returns (code, {kernel name: (launches, total_ms, layers covered)})."""
    arr = (KvpKernelStat * len(KERNEL_KINDS))()
    rc = lib().kvp_profile_read(handle, arr)
    return rc, {name: (arr[i].launches, arr[i].total_ms, arr[i].layers) for i, name in enumerate(KERNEL_KINDS)}


def kvp_probe_mfma(device_out, out_bytes, workgroups, iters, stream=0):
    """Returns (code, flops of the launch)."""
    flops = ctypes.c_double()
    rc = lib().kvp_probe_mfma(device_out, out_bytes, workgroups, iters, stream, ctypes.byref(flops))
    return rc, flops.value


def kvp_probe_copy(device_dst, device_src, nbytes, workgroups, stream=0):
    return lib().kvp_probe_copy(device_dst, device_src, nbytes, workgroups, stream)


def kvp_free_cache(handle):
    lib().kvp_free_cache(handle)


# ---- convenience holder --------------------------------------------------------
def _check(rc, what):
    if rc != KVP_OK:
        raise KvpError(rc, what)


class Cache:
    """Owns the device buffer (a torch uint8 tensor) and forwards calls.

    Tensors must be contiguous bfloat16 on the cache's device.  Every method is
    argument marshalling around one C call."""

    # bytes of guard band on either side of the device buffer of every Cache created from now on
    # (tests set it; see guards_intact)
    default_guard_bytes = 0

    def __init__(self, n_layers, n_q_heads, n_kv_heads, head_dim, budget, chunk_max, segments,
                 merge=False, scratch_sets=1, softmax_scale=0.0, device="cuda:0", stream=None,
                 guard_bytes=None):
        import torch
        self.torch = torch
        self.cfg = KvpConfig(n_layers, n_q_heads, n_kv_heads, head_dim, budget, chunk_max,
                             int(merge), scratch_sets, 0, softmax_scale)
        self.segments = list(segments)
        nbytes = kvp_cache_bytes(self.cfg)
        if nbytes == 0:
            raise KvpError(KVP_EINVAL, "kvp_cache_bytes")
        self.device = torch.device(device)
        self.nbytes = nbytes
        self.persistent_bytes = kvp_persistent_bytes(self.cfg)
        # Optional guard bands: the whole allocation is filled with 0xFF (a NaN pattern in bf16 and
        # fp32, -1 as a token index) before the library gets the part in the middle, so that a
        # write outside that part shows up in guards_intact() and a read of a never-written slot
        # shows up as NaN in the results.
        self.guard = Cache.default_guard_bytes if guard_bytes is None else int(guard_bytes)
        assert self.guard >= 0 and self.guard % 256 == 0
        self.buf = torch.empty(nbytes + 256 + 2 * self.guard, dtype=torch.uint8, device=self.device)
        if self.guard:
            self.buf.fill_(0xFF)
            if stream is not None:      # the fill ran on torch's current stream, the library may use another
                torch.cuda.current_stream(self.device).synchronize()
        self._base = (self.buf.data_ptr() + self.guard + 255) // 256 * 256
        rc, self.handle = kvp_init_cache(self.cfg, self.segments, self._base, nbytes, self._stream(stream))
        _check(rc, "kvp_init_cache")

    def guards_intact(self):
        """True when no byte outside the part handed to the library has changed since creation
        (always True for a cache created without guard bands)."""
        if not self.guard:
            return True
        lo = self._base - self.buf.data_ptr()
        hi = lo + self.nbytes
        return bool((self.buf[:lo] == 0xFF).all()) and bool((self.buf[hi:] == 0xFF).all())

    def _stream(self, stream=None):
        if stream is None:
            stream = self.torch.cuda.current_stream(self.device)
        return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)

    def _ptr(self, t, dtype):
        assert t.is_contiguous() and t.dtype == dtype and t.device == self.device, (t.dtype, t.device)
        return t.data_ptr()

    def prefill_chunk(self, layer, token_begin, q, k, v, out=None, stream=None):
        bf = self.torch.bfloat16
        n = q.shape[0]
        assert q.shape == (n, self.cfg.n_q_heads, self.cfg.head_dim)
        assert k.shape == v.shape == (n, self.cfg.n_kv_heads, self.cfg.head_dim)
        if out is None:
            out = self.torch.empty_like(q)
        assert out.shape == q.shape
        rc = kvp_prefill_chunk(self.handle, layer, token_begin, n, self._ptr(q, bf), self._ptr(k, bf),
                               self._ptr(v, bf), self._ptr(out, bf), self._stream(stream))
        _check(rc, "kvp_prefill_chunk")
        return out

    def prefill_chunk_keydiff(self, layer, token_begin, q, k, v, out=None, stream=None):
        bf = self.torch.bfloat16
        n = q.shape[0]
        assert q.shape == (n, self.cfg.n_q_heads, self.cfg.head_dim)
        assert k.shape == v.shape == (n, self.cfg.n_kv_heads, self.cfg.head_dim)
        if out is None:
            out = self.torch.empty_like(q)
        assert out.shape == q.shape
        rc = kvp_prefill_chunk_keydiff(self.handle, layer, token_begin, n, self._ptr(q, bf), self._ptr(k, bf),
                                       self._ptr(v, bf), self._ptr(out, bf), self._stream(stream))
        _check(rc, "kvp_prefill_chunk_keydiff")
        return out

    def decode_step(self, layer, q, k_tail, v_tail, out=None, stream=None):
        """q [Hq, d]; k_tail, v_tail [n_tail, Hkv, d] (the generated tokens, the current one last)."""
        bf = self.torch.bfloat16
        assert q.shape == (self.cfg.n_q_heads, self.cfg.head_dim)
        n_tail = k_tail.shape[0]
        assert k_tail.shape == v_tail.shape == (n_tail, self.cfg.n_kv_heads, self.cfg.head_dim)
        if out is None:
            out = self.torch.empty_like(q)
        assert out.shape == q.shape
        rc = kvp_decode_step(self.handle, layer, self._ptr(q, bf), self._ptr(k_tail, bf), self._ptr(v_tail, bf),
                             n_tail, self._ptr(out, bf), self._stream(stream))
        _check(rc, "kvp_decode_step")
        return out

    def decode_step_static(self, layer, q, k_tail, v_tail, out, stream=None):
        """decode_step with the library's static scratch; `out` must be given (nothing is allocated)."""
        bf = self.torch.bfloat16
        assert q.shape == out.shape == (self.cfg.n_q_heads, self.cfg.head_dim)
        n_tail = k_tail.shape[0]
        assert k_tail.shape == v_tail.shape == (n_tail, self.cfg.n_kv_heads, self.cfg.head_dim)
        rc = kvp_decode_step_static(self.handle, layer, self._ptr(q, bf), self._ptr(k_tail, bf), self._ptr(v_tail, bf),
                                    n_tail, self._ptr(out, bf), self._stream(stream))
        _check(rc, "kvp_decode_step_static")
        return out

    def prefill_chunk_proxy(self, layer, token_begin, q, k, v, q_obs, out=None, stream=None):
        bf = self.torch.bfloat16
        n = q.shape[0]
        assert q.shape == (n, self.cfg.n_q_heads, self.cfg.head_dim)
        assert k.shape == v.shape == (n, self.cfg.n_kv_heads, self.cfg.head_dim)
        assert q_obs.shape[1:] == q.shape[1:]
        if out is None:
            out = self.torch.empty_like(q)
        assert out.shape == q.shape
        rc = kvp_prefill_chunk_proxy(self.handle, layer, token_begin, n, self._ptr(q, bf), self._ptr(k, bf),
                                     self._ptr(v, bf), self._ptr(out, bf), self._ptr(q_obs, bf),
                                     q_obs.shape[0], self._stream(stream))
        _check(rc, "kvp_prefill_chunk_proxy")
        return out

    def compact(self, layer, scores_override=None, stream=None):
        ptr = None
        if scores_override is not None:
            ptr = self._ptr(scores_override, self.torch.float32)
        _check(kvp_compact(self.handle, layer, ptr, self._stream(stream)), "kvp_compact")

    def compact_layers(self, first_layer, n_layers, stream=None):
        _check(kvp_compact_layers(self.handle, first_layer, n_layers, self._stream(stream)), "kvp_compact_layers")

    def _view_tensor(self, ptr, shape, dtype):
        """A tensor aliasing part of the device buffer."""
        torch = self.torch
        off = ptr - self.buf.data_ptr()
        numel = 1
        for s in shape:
            numel *= s
        nbytes = numel * torch.empty((), dtype=dtype).element_size()
        assert 0 <= off and off + nbytes <= self.buf.numel()
        return self.buf[off:off + nbytes].view(dtype).view(*shape)

    def decode_ready(self, layer):
        """(k, v, token_idx, weight, count, next_token): tensors alias the cache."""
        torch = self.torch
        rc, vw = kvp_decode_ready(self.handle, layer)
        _check(rc, "kvp_decode_ready")
        h, m, d = self.cfg.n_kv_heads, self.cfg.budget, self.cfg.head_dim
        return (self._view_tensor(vw.k, (h, m, d), torch.bfloat16),
                self._view_tensor(vw.v, (h, m, d), torch.bfloat16),
                self._view_tensor(vw.token_idx, (h, m), torch.int32),
                self._view_tensor(vw.weight, (h, m), torch.float32),
                vw.count, vw.next_token)

    def set_state(self, layer, count, next_token):
        _check(kvp_set_state(self.handle, layer, count, next_token), "kvp_set_state")

    def set_attention_shape(self, shape):
        _check(kvp_set_attention_shape(self.handle, shape), "kvp_set_attention_shape")

    def set_deferred_scoring(self, on):
        _check(kvp_set_deferred_scoring(self.handle, on), "kvp_set_deferred_scoring")

    def set_score_sweep(self, fused):
        _check(kvp_set_score_sweep(self.handle, fused), "kvp_set_score_sweep")

    def debug_last(self, layer):
        """(scores, keep, dst) of the layer's last block, each [Hkv, n_cand]."""
        torch = self.torch
        rc, s, k, d, n, st = kvp_debug_last(self.handle, layer)
        _check(rc, "kvp_debug_last")
        h = self.cfg.n_kv_heads
        return (self._view_tensor(s, (h, st), torch.float32)[:, :n],
                self._view_tensor(k, (h, st), torch.uint8)[:, :n],
                self._view_tensor(d, (h, st), torch.int32)[:, :n])

    def totals(self):
        """{name: count} of the compaction totals since creation (synchronises the device)."""
        rc, p = kvp_debug_totals(self.handle)
        _check(rc, "kvp_debug_totals")
        self.torch.cuda.synchronize(self.device)
        t = self._view_tensor(p, (len(TOTALS),), self.torch.int64).cpu().tolist()
        return dict(zip(TOTALS, t))

    def profile_enable(self, on=True):
        _check(kvp_profile_enable(self.handle, on), "kvp_profile_enable")

    def profile_read(self):
        rc, stats = kvp_profile_read(self.handle)
        _check(rc, "kvp_profile_read")
        return stats

    def close(self):
        if getattr(self, "handle", None):
            kvp_free_cache(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
