"""GPU parity of the unfused comparison path (accumulated attention weights; Fig. 1, Sec. 4.1)
against the oracle's accumulated-attention rule, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2603_11504_amd import longflow as lf
from paper_2603_11504_amd import workloads as W

from parity import run_lockstep

pytestmark = pytest.mark.gpu

UNF = lf.LF_FLAG_UNFUSED_ACCUM
RULE = "accumulated_attention"


def _wl(name, B, Hq, Hkv, N, n_init=0, steps=0, **kw):
    return W.Workload(name, "bf16", B, Hq, Hkv, 128, N, n_init, steps or 2 * N, **kw)


@pytest.mark.parametrize("B,Hq,Hkv,N,extra", [
    (3, 1, 1, 61, 0), (3, 14, 2, 129, 0), (2, 7, 1, 1000, 0), (2, 16, 1, 300, 0), (1, 10, 2, 2100, 0),
    (2, 7, 1, 1000, lf.LF_FLAG_FORCE_SPLIT), (2, 8, 2, 515, lf.LF_FLAG_FORCE_UNIT),
], ids=lambda v: str(v))
def test_fill_then_evict_every_step(B, Hq, Hkv, N, extra):
    wl = _wl(f"unf_{Hq}x{Hkv}_n{N}", B, Hq, Hkv, N, steps=N + 60, sink_scale=4.0, seed=500 + N)
    rep, gpu, _ = run_lockstep(wl, flags=UNF | extra, rule=RULE, check_scores_every=53)
    print(f"\nunfused {Hq}x{Hkv} n{N}: decisions {rep.decisions} near-ties {rep.near_ties} "
          f"max|dout| {rep.max_out_err:.2e} max acc rel {rep.max_score_rel:.2e}")
    assert rep.steps == N + 60
    # the near-tie allowance is for rare cases, not a licence
    assert rep.near_ties <= max(2, rep.decisions // 200)


def test_prefilled_rows_start_at_zero_and_long_runs_stay_in_step():
    wl = _wl("unf_prefilled", 2, 28, 4, 2048, n_init=2000, steps=600, sink_scale=4.0, seed=9)
    rep, gpu, ora = run_lockstep(wl, flags=UNF, rule=RULE, check_scores_every=100)
    print(f"\nunfused prefilled: decisions {rep.decisions} near-ties {rep.near_ties} max acc rel {rep.max_score_rel:.2e}")
    assert rep.steps == 600
    assert rep.near_ties <= 4


def test_cfg2_geometry_full_size_sampled_units():
    wl = W.CONFIGS[2]
    units = np.arange(0, wl.units, 8)
    rep, gpu, _ = run_lockstep(wl, steps=4, host_inputs=False, units=units, flags=UNF, rule=RULE,
                               check_scores_every=3)
    print(f"\nunfused cfg2: decisions {rep.decisions} near-ties {rep.near_ties} max|dout| {rep.max_out_err:.2e}")
    assert rep.steps == 4


def test_cfg3_geometry_one_layer_full_size_sampled_units():
    wl = W.CONFIGS[3]
    rng = np.random.default_rng(5)
    units = np.sort(rng.choice(wl.units, size=16, replace=False))
    rep, gpu, _ = run_lockstep(wl, steps=3, host_inputs=False, units=units, flags=UNF, rule=RULE,
                               check_scores_every=2)
    print(f"\nunfused cfg3: decisions {rep.decisions} near-ties {rep.near_ties} max|dout| {rep.max_out_err:.2e}")
    gpu.close()
    del gpu
    torch.cuda.empty_cache()


def test_attention_output_equals_the_plain_attention_kernel_bitwise():
    """Step 2 of the unfused path IS the attention-only kernel: same bits on the same cache."""
    wl = _wl("unf_vs_plain", 4, 28, 4, 700, n_init=700, steps=1, seed=31)
    k0, v0 = W.device_prefill(wl, "cuda")
    q, k, v = W.device_step(wl, 0, "cuda")
    unf = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, 128, wl.budget, flags=UNF, k_init=k0, v_init=v0)
    unf.set_pending(torch.full((wl.batch, wl.kv_heads), 13, dtype=torch.int32))
    out_u, idx_u = unf.decode_step(q, k, v)
    torch.cuda.synchronize()
    # the same rows, with slot 13 already replaced, through the attention-only cache
    k1, v1 = k0.clone(), v0.clone()
    k1[:, :, 13] = k
    v1[:, :, 13] = v
    plain = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, 128, wl.budget, flags=lf.LF_FLAG_ATTENTION_ONLY,
                             k_init=k1, v_init=v1)
    out_p, _ = plain.decode_step(q)
    torch.cuda.synchronize()
    assert torch.equal(out_u.view(torch.int16), out_p.view(torch.int16))
    assert torch.equal(unf.k_cache.view(torch.int16), k1.view(torch.int16))
    assert torch.equal(unf.v_cache.view(torch.int16), v1.view(torch.int16))
    # one step of weights on empty books: every unit's accumulators sum to the group size
    acc = unf.scores()
    np.testing.assert_allclose(acc.sum(-1).cpu().numpy(), wl.group, rtol=2e-5)
    assert (acc[:, :, 13] > 0).all()


def test_unsupported_combinations_are_refused():
    with pytest.raises(lf.LongFlowError):
        lf.LongFlowCache(1, 4, 1, 64, 128, flags=UNF)                                  # head_dim 64
    with pytest.raises(lf.LongFlowError):
        lf.LongFlowCache(1, 4, 1, 128, 128, dtype=torch.float32, flags=UNF)            # fp32
    with pytest.raises(lf.LongFlowError):
        lf.LongFlowCache(1, 4, 1, 128, 128, flags=UNF | lf.LF_FLAG_ATTENTION_ONLY)
    c = lf.LongFlowCache(1, 4, 1, 128, 128, flags=UNF)
    with pytest.raises(lf.LongFlowError):
        c.set_mask(torch.ones(1, 1, 128))
    with pytest.raises(lf.LongFlowError):
        c.scores()                                                                     # before the first step
    with pytest.raises(lf.LongFlowError):
        lf.LongFlowGroup([c])
    q = torch.randn(1, 4, 128, device="cuda", dtype=torch.bfloat16)
    kv = torch.randn(1, 1, 128, device="cuda", dtype=torch.bfloat16)
    c.decode_step(q, kv, kv)
    with pytest.raises(lf.LongFlowError):
        c.evict_lowest(2)
    info = lf.longflow_plan_info(c.cfg)
    assert info.launches_per_step >= 4
    torch.cuda.synchronize()


def test_unfused_steps_replayed_from_a_hip_graph_match_eager():
    # the four launches of a step are plain kernels: a caller may capture steady-state steps
    wl = _wl("unf_graph", 4, 28, 4, 1024, n_init=1023, steps=8, seed=72)
    k0, v0 = W.host_prefill(wl)
    mk = lambda: lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, flags=UNF,
                                  k_init=W.to_torch(k0, wl, "cuda"), v_init=W.to_torch(v0, wl, "cuda"))
    eager, graphed = mk(), mk()
    qs, ks, vs = (torch.empty_like(W.to_torch(x, wl, "cuda")) for x in W.host_step(wl, 0))
    for t in range(2):
        for dst, src in zip((qs, ks, vs), W.host_step(wl, t)):
            dst.copy_(W.to_torch(src, wl, "cuda"))
        eager.decode_step(qs, ks, vs)
        graphed.decode_step(qs, ks, vs)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.decode_step(qs, ks, vs)
    for t in range(2, 8):
        for dst, src in zip((qs, ks, vs), W.host_step(wl, t)):
            dst.copy_(W.to_torch(src, wl, "cuda"))
        o_e, i_e = eager.decode_step(qs, ks, vs)
        o_e, i_e = o_e.clone(), i_e.clone()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_e.view(torch.int16), graphed.out.view(torch.int16)), f"replay {t}"
        assert torch.equal(i_e, graphed.evict_idx), f"replay {t}"
        junk = torch.randn(1 << 20, device="cuda").sum().item()
        assert junk == junk
    assert torch.equal(eager.scores(), graphed.scores())
    assert torch.equal(eager.k_cache.view(torch.int16), graphed.k_cache.view(torch.int16))


def test_degenerate_budgets_of_a_few_slots():
    for N in (1, 2, 3, 15, 16, 17):
        wl = _wl(f"unf_tiny_{N}", 2, 6, 2, N, steps=N + 12, sink_scale=4.0, seed=300 + N)
        rep, gpu, _ = run_lockstep(wl, flags=UNF, rule=RULE, check_scores_every=1)
        assert rep.steps == N + 12
