"""The batch eviction that allocates nothing (longflow_evict_lowest_static), through the C ABI,
against longflow_evict_lowest on a twin cache: same dropped slots in the same order, same cache
bits, same validity, and the same steps afterwards.  Two calls in a row share the library's
built-in scratch array; the second is the smaller one, so stale entries of the first lie
behind it."""
import ctypes

import pytest
import torch

from paper_2603_11504_amd import longflow as lf
from paper_2603_11504_amd import workloads as W

pytestmark = pytest.mark.gpu


def _twins(wl, flags=0):
    k0, v0 = W.host_prefill(wl)
    mk = lambda: lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, dtype=W.torch_dtype(wl),
                                  flags=flags, k_init=W.to_torch(k0, wl, "cuda"), v_init=W.to_torch(v0, wl, "cuda"))
    return mk(), mk()


def _step_both(wl, a, b, t, view):
    q, k, v = (W.to_torch(x, wl, "cuda") for x in W.host_step(wl, t))
    oa, ia = a.decode_step(q, k, v)
    ob, ib = b.decode_step(q, k, v)
    torch.cuda.synchronize()
    assert torch.equal(oa.view(view), ob.view(view)) and torch.equal(ia, ib), f"{wl.name} step {t}"


def _evict_both_ways(wl, k, flags=0):
    view = torch.int16 if wl.dtype == "bf16" else torch.int32
    a, b = _twins(wl, flags)
    for t in range(4):
        _step_both(wl, a, b, t, view)
    ev_a = a.evict_lowest(k)                      # scratch buffer passed in
    ev_b = torch.full((wl.batch, wl.kv_heads, k), -7, dtype=torch.int32, device="cuda")
    free_before = torch.cuda.memory_allocated()
    rc = lf.lib().longflow_evict_lowest_static(b._h, k, ctypes.c_void_p(ev_b.data_ptr()),
                                               ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == lf.LF_OK, lf.lib().longflow_last_error().decode()
    assert torch.cuda.memory_allocated() == free_before
    torch.cuda.synchronize()
    assert torch.equal(ev_a, ev_b), f"{wl.name}: dropped slots differ"
    assert torch.equal(a.mask(), b.mask())
    assert torch.equal(a.k_cache.view(view), b.k_cache.view(view)) and torch.equal(a.v_cache.view(view), b.v_cache.view(view))
    assert a.valid_count == b.valid_count == wl.budget
    holes = int((a.mask() == 0).reshape(wl.units, -1).sum(-1).max())   # k dropped slots, plus those never filled
    for t in range(4, 4 + holes + 3):             # the holes refill, then per-step eviction resumes
        _step_both(wl, a, b, t, view)
    assert bool(a.mask().all()) and bool(b.mask().all())
    a.close(); b.close()


def test_static_scratch_eviction_equals_the_one_with_a_scratch_argument_twice_in_a_row():
    big = W.Workload("noalloc_big", "bf16", 8, 16, 4, 128, 2048, 2047, 1, sink_scale=4.0, seed=401)     # 65536 slots
    small = W.Workload("noalloc_small", "bf16", 2, 8, 2, 128, 300, 299, 1, sink_scale=4.0, seed=402)    # 1200 slots
    _evict_both_ways(big, 37)
    _evict_both_ways(small, 5)
    # the vector-ALU family (fp32) goes through the same two kernels
    _evict_both_ways(W.Workload("noalloc_f32", "f32", 2, 8, 2, 64, 200, 150, 1, sink_scale=4.0, seed=403), 11)


def test_static_scratch_eviction_refuses_what_does_not_fit():
    n = lf.LF_EVICT_STATIC_MAX_SLOTS + 16
    z = torch.zeros((1, 1, 16, 128), dtype=torch.bfloat16, device="cuda")
    c = lf.LongFlowCache(1, 2, 1, 128, n, k_init=z, v_init=z)
    with pytest.raises(lf.LongFlowError) as e:
        c.evict_lowest_static(3)
    assert e.value.status == lf.LF_ERR_WORKSPACE and "scratch" in str(e.value)
    assert c.valid_count == 16
    c.close()
    # at the limit itself the size check passes (the next check, "no step yet", answers)
    c = lf.LongFlowCache(1, 2, 1, 128, lf.LF_EVICT_STATIC_MAX_SLOTS, k_init=z, v_init=z)
    with pytest.raises(lf.LongFlowError) as e:
        c.evict_lowest_static(3)
    assert e.value.status == lf.LF_ERR_STATE
    c.close()
