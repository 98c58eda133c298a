"""Seeded generator of one layer's Q, K, V for a workload.

Recipe (one ``numpy.random.default_rng(seed0 + layer)`` per layer; the draw
order below is part of the recipe):

for each segment in prefix order
  visual segment, K then V, each ``[n_tokens, Hkv, d]``:
    per field unit (every plane, or one unit shared by all planes), per KV
    head and channel: four sinusoids with frequencies ``fy, fx ~ U[0, 2)``
    cycles per grid and phase ``phi ~ U[0, 2 pi)``,
    ``F(y, x) = sum_m a sin(2 pi (fy_m y / gh + fx_m x / gw) + phi_m)``,
    ``a = 1/sqrt(2)`` so that F has unit variance;
    shared-field (video) workloads add a per-plane offset following an AR(1)
    process with correlation 0.9 and stationary deviation 0.5;
    then i.i.d. noise of deviation 0.1 on every element.
  text segment: K then V, standard normal.
finally Q ``[N, Hq, d]``, standard normal for every position.

Everything is rounded once to bfloat16 (round-to-nearest-even) and returned
as uint16 bit patterns; these bits are what every consumer reads.
"""
import numpy as np

from .configs import VISUAL, Workload

FIELD_TERMS = 4
FIELD_AMPLITUDE = 1.0 / np.sqrt(2.0)
NOISE_STD = 0.1
OFFSET_STD = 0.5
OFFSET_CORR = 0.9


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even.
    Inputs are finite; NaN payloads are not preserved."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _visual_tensor(rng: np.random.Generator, seg, n_kv_heads: int, d: int, field_unit: str) -> np.ndarray:
    gh, gw, planes = seg.grid_h, seg.grid_w, seg.n_planes
    units = planes if field_unit == "plane" else 1
    shape = (units, n_kv_heads, d, FIELD_TERMS)
    fy = rng.uniform(0.0, 2.0, size=shape)
    fx = rng.uniform(0.0, 2.0, size=shape)
    phi = rng.uniform(0.0, 2.0 * np.pi, size=shape)
    y = (np.arange(gh, dtype=np.float64) / gh)[:, None]
    x = (np.arange(gw, dtype=np.float64) / gw)[None, :]
    # field[u, y, x, h, c]
    field = np.zeros((units, gh, gw, n_kv_heads, d), dtype=np.float64)
    for m in range(FIELD_TERMS):
        arg = 2.0 * np.pi * (
            fy[:, None, None, :, :, m] * y[None, :, :, None, None]
            + fx[:, None, None, :, :, m] * x[None, :, :, None, None]
        ) + phi[:, None, None, :, :, m]
        field += FIELD_AMPLITUDE * np.sin(arg)
    if field_unit == "plane":
        vals = field.astype(np.float32)                       # [planes, gh, gw, h, c]
    else:
        o = np.empty((planes, n_kv_heads, d), dtype=np.float64)
        o[0] = OFFSET_STD * rng.standard_normal((n_kv_heads, d))
        innov = np.sqrt(1.0 - OFFSET_CORR ** 2) * OFFSET_STD
        eps = rng.standard_normal((max(planes - 1, 0), n_kv_heads, d))
        for t in range(1, planes):
            o[t] = OFFSET_CORR * o[t - 1] + innov * eps[t - 1]
        vals = (field[0][None] + o[:, None, None, :, :]).astype(np.float32)
    vals = vals.reshape(planes * gh * gw, n_kv_heads, d)
    noise = rng.standard_normal(vals.shape, dtype=np.float32)
    return vals + np.float32(NOISE_STD) * noise


def layer_inputs(wl: Workload, layer: int, seed0: int = 0):
    """Q, K, V of one layer as bf16 bit patterns: ``q [N, Hq, d]``,
    ``k, v [N, Hkv, d]`` (uint16, C-contiguous)."""
    rng = np.random.default_rng(seed0 + layer)
    n, hq, hkv, d = wl.n_tokens, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    k = np.empty((n, hkv, d), dtype=np.float32)
    v = np.empty((n, hkv, d), dtype=np.float32)
    for seg in wl.segments:
        lo, hi = seg.token_begin, seg.token_begin + seg.n_tokens
        if seg.kind == VISUAL:
            k[lo:hi] = _visual_tensor(rng, seg, hkv, d, wl.field_unit)
            v[lo:hi] = _visual_tensor(rng, seg, hkv, d, wl.field_unit)
        else:
            k[lo:hi] = rng.standard_normal((seg.n_tokens, hkv, d), dtype=np.float32)
            v[lo:hi] = rng.standard_normal((seg.n_tokens, hkv, d), dtype=np.float32)
    q = rng.standard_normal((n, hq, d), dtype=np.float32)
    return f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v)
