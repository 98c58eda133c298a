"""kvp_decode_step_static: the decode step whose partial results live in the library's
file-scope device array instead of the cache's scratch set (for callers that cannot allocate
or lend memory).  Checked against kvp_decode_step and against the oracle, on two calls in a
row that share the array, the second smaller than the first.  Collected last on purpose."""
import numpy as np
import pytest
import torch

import paper_2604_16734_amd as K
from kvp_workload import Segment, f32_to_bf16_bits
from oracle import kvp_oracle as O
from tests import gpu_util as U

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bits(rng, shape, scale=1.0):
    return f32_to_bf16_bits((scale * rng.standard_normal(shape)).astype(np.float32))


def _load(cache, layer, rng, hkv, d, budget, c):
    oc = O.LayerCache(hkv, d, budget)
    kb, vb = _bits(rng, (c, hkv, d)), _bits(rng, (c, hkv, d))
    oc.compact(0, O.bf16_bits_to_f64(kb), O.bf16_bits_to_f64(vb), np.zeros((hkv, c), dtype=np.float32))
    U.upload_state(cache, layer, oc)
    cache.set_state(layer, c, c)
    return oc


def _step_both_ways(cache, layer, oc, rng, hq, hkv, d, n_tail):
    qb, kb, vb = _bits(rng, (hq, d), 2.0), _bits(rng, (n_tail, hkv, d)), _bits(rng, (n_tail, hkv, d))
    _, _, k_all, v_all = oc.candidates(oc.count, O.bf16_bits_to_f64(kb), O.bf16_bits_to_f64(vb))
    ref = O.decode_step(O.bf16_bits_to_f64(qb), k_all, v_all)
    q, kt, vt = U.bits_to_torch(qb), U.bits_to_torch(kb), U.bits_to_torch(vb)
    out_static = torch.full((hq, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    print("kvp_decode_step_static: count", oc.count, "n_tail", n_tail, flush=True)
    cache.decode_step_static(layer, q, kt, vt, out_static)
    out_plain = cache.decode_step(layer, q, kt, vt)
    torch.cuda.synchronize()
    assert U.out_rel_err(U.torch_bf16_to_f64(out_static), ref) <= U.OUT_TOL
    # the same kernels, the same number of workgroups per KV head, a fixed fold order: the same bits
    assert torch.equal(out_static.view(torch.int16), out_plain.view(torch.int16))
    return out_static


def test_static_scratch_decode_step_two_calls_second_smaller():
    hq, hkv, d, budget = 32, 8, 128, 2048
    rng = np.random.default_rng(77)
    cache = K.Cache(2, hq, hkv, d, budget, 1024, [Segment(0, 100000, 0)], scratch_sets=1, device=DEV)
    big = _load(cache, 0, rng, hkv, d, budget, 2048)
    first = _step_both_ways(cache, 0, big, rng, hq, hkv, d, n_tail=70)        # 34 workgroups per KV head
    small = _load(cache, 1, rng, hkv, d, budget, 150)
    _step_both_ways(cache, 1, small, rng, hq, hkv, d, n_tail=1)                # 3: most of the array keeps the first call's data
    again = _step_both_ways(cache, 1, small, rng, hq, hkv, d, n_tail=3)
    assert again.shape == first.shape
    cache.close()


def test_static_scratch_decode_step_does_not_need_the_scratch_set():
    hq, hkv, d, budget = 8, 2, 64, 256
    rng = np.random.default_rng(78)
    cache = K.Cache(2, hq, hkv, d, budget, 64, [Segment(0, 100000, 0)], scratch_sets=1, device=DEV)
    oc = _load(cache, 1, rng, hkv, d, budget, 200)
    qb, kb, vb = _bits(rng, (hq, d), 2.0), _bits(rng, (2, hkv, d)), _bits(rng, (2, hkv, d))
    _, _, k_all, v_all = oc.candidates(oc.count, O.bf16_bits_to_f64(kb), O.bf16_bits_to_f64(vb))
    ref = O.decode_step(O.bf16_bits_to_f64(qb), k_all, v_all)
    q, kt, vt = U.bits_to_torch(qb), U.bits_to_torch(kb), U.bits_to_torch(vb)
    # layer 0 takes the only scratch set: a block of it is pending
    blk = [U.bits_to_torch(_bits(rng, (16, h, d))) for h in (hq, hkv, hkv)]
    cache.prefill_chunk(0, 0, *blk)
    out = torch.empty((hq, d), dtype=torch.bfloat16, device=DEV)
    assert K.kvp_decode_step(cache.handle, 1, q.data_ptr(), kt.data_ptr(), vt.data_ptr(), 2, out.data_ptr()) == K.KVP_ESTATE
    cache.decode_step_static(1, q, kt, vt, out)
    cache.compact(0)
    torch.cuda.synchronize()
    assert U.out_rel_err(U.torch_bf16_to_f64(out), ref) <= U.OUT_TOL
    cache.close()
