"""GPU parity of the bulk fill (longflow_fill_steps) against the oracle: T tokens at once must
give what T consecutive decode steps give."""
import numpy as np
import pytest
import torch

from oracle import longflow_oracle as oracle
from paper_2603_11504_amd import longflow as lf
from paper_2603_11504_amd import workloads as W

from parity import OUT_TOL, ParityReport, compare_indices, run_lockstep

pytestmark = pytest.mark.gpu


def _wl(name, dtype, B, Hq, Hkv, D, N, n_init=0, **kw):
    return W.Workload(name, dtype, B, Hq, Hkv, D, N, n_init, 4 * N, **kw)


def _stack_steps(wl, t0, T, device="cuda"):
    per = [W.device_step(wl, t, device) for t in range(t0, t0 + T)]
    return tuple(torch.stack([x[i] for x in per]).contiguous() for i in range(3))


def _fill_and_compare(wl, chunks, units=None, flags=0, tail_steps=8, k_scale=None, out_tol=None):
    """Prefill both sides, feed the chunks through fill_steps / oracle.fill, compare everything,
    then continue with ordinary lock-step decode steps (evicting once full)."""
    dt = W.torch_dtype(wl)
    G, D, N = wl.group, wl.head_dim, wl.budget
    all_units = np.arange(wl.units) if units is None else np.asarray(units)
    nu = len(all_units)
    sel = torch.as_tensor(all_units, device="cuda")
    k0, v0 = W.device_prefill(wl, "cuda")
    gpu = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, D, N, dtype=dt, flags=flags, k_init=k0, v_init=v0)
    ora = oracle.OracleCache(nu, G, 1, D, N)
    if wl.n_init:
        ora.init(W.to_f64(k0.reshape(wl.units, wl.n_init, D)[sel].reshape(nu, 1, wl.n_init, D)),
                 W.to_f64(v0.reshape(wl.units, wl.n_init, D)[sel].reshape(nu, 1, wl.n_init, D)))
    else:
        ora.init()
    rep = ParityReport()
    t = 0
    for T in chunks:
        q, k, v = _stack_steps(wl, t, T)
        for tok, f in (k_scale or {}).items():   # keys of some tokens made large (power of two: exact in storage)
            if t <= tok < t + T:
                k[tok - t] *= f
        out_t, idx_t = gpu.fill_steps(q, k, v)
        torch.cuda.synchronize()
        o_ref, i_ref = ora.fill(W.to_f64(q.reshape(T, wl.units, G, D)[:, sel]),
                                W.to_f64(k.reshape(T, wl.units, 1, D)[:, sel]),
                                W.to_f64(v.reshape(T, wl.units, 1, D)[:, sel]))
        o_gpu = W.to_f64(out_t.reshape(T, wl.units, G, D)[:, sel])
        assert np.isfinite(o_gpu).all()
        err = float(np.abs(o_gpu - o_ref).max())
        rep.max_out_err = max(rep.max_out_err, err)
        assert err <= (out_tol or OUT_TOL[wl.dtype]), f"chunk at t={t} of {T}: max |out - oracle| = {err:.3e}"
        t += T
        assert gpu.valid_count == ora.count == min(N, wl.n_init + t)
        i_gpu = idx_t.reshape(-1)[sel].cpu().numpy()
        full = np.full(nu, ora.count == N)
        if compare_indices(i_gpu, i_ref, ora.scores(), full, rep, where=f"{wl.name} after {t} tokens"):
            ora.set_pending(i_gpu.reshape(nu, 1))
        # the rows are where sequential steps would have put them, bit for bit
        Ko, Vo = ora.kv()
        n = ora.count
        Kg = W.to_f64(gpu.k_cache.reshape(wl.units, N, D)[sel][:, :n])
        Vg = W.to_f64(gpu.v_cache.reshape(wl.units, N, D)[sel][:, :n])
        assert np.array_equal(Kg, Ko.reshape(nu, N, D)[:, :n]) and np.array_equal(Vg, Vo.reshape(nu, N, D)[:, :n])
        s_gpu = gpu.scores().reshape(wl.units, N)[sel].cpu().numpy().astype(np.float64)
        s_ref = ora.scores().reshape(nu, N)
        rel = np.abs(s_gpu[:, :n] - s_ref[:, :n]) / np.maximum(s_ref[:, :n], 1e-30)
        assert ((rel <= 1e-5) | (s_ref[:, :n] < 1e-35)).all() and (s_gpu[:, n:] == 0).all()
    if tail_steps:
        run_lockstep(wl, steps=tail_steps, units=units, gpu_cache=gpu, oracle_cache=ora, t0=t, report=rep,
                     host_inputs=False, check_scores_every=3)
    return rep, gpu, ora


@pytest.mark.parametrize("Hq,Hkv,N,n_init,chunks", [
    (28, 4, 700, 0, [1, 2, 5, 300, 391, 1]),          # G = 7: 2 tokens per product; ends exactly full
    (8, 2, 515, 17, [100, 33, 365]),                  # G = 4, ragged budget, ends full
    (3, 3, 130, 1, [129]),                            # G = 1: 16 tokens per product, one chunk to the brim
    (16, 1, 300, 40, [64, 64, 64]),                   # G = 16: one token per product; stays short of full
    (10, 2, 2100, 2000, [7, 50, 43]),                 # G = 5 (3 tokens, one column idle), long prefix
    (14, 2, 257, 0, [16, 15, 17, 48, 161]),           # tile-edge chunk sizes
], ids=lambda v: str(v).replace(" ", ""))
def test_bulk_fill_matches_the_oracle(Hq, Hkv, N, n_init, chunks):
    wl = _wl(f"fill_{Hq}x{Hkv}_n{N}", "bf16", 3, Hq, Hkv, 128, N, n_init=n_init, sink_scale=4.0, seed=900 + N)
    rep, gpu, ora = _fill_and_compare(wl, chunks)
    print(f"\nfill {Hq}x{Hkv} n{N}: decisions {rep.decisions} near-ties {rep.near_ties} max|dout| {rep.max_out_err:.2e}")


def test_bulk_fill_reference_raised_in_either_tile_of_a_pair():
    # The batched kernel takes two tiles per P V product and keeps the first tile's weights pending while the
    # second may still raise the softmax reference.  Keys 8x the usual size put logits far above everything
    # before them into second tiles of pairs (tokens 19, 53, 150), into first tiles (100, 131) and into both
    # tiles of one pair (192, 210): every order of "raise" and "pending weights" occurs for many columns.
    wl = _wl("fill_raise", "bf16", 2, 28, 4, 128, 400, n_init=0, seed=77)
    # A dominant token makes an output close to one value row, whose entries reach magnitude 4: bf16 numbers are
    # 2^-6 apart there, and the output may be off by half a step for its own rounding plus a step for the single
    # bf16 weight of the dominant token (the interface says so): 1.5 * 2^-6 = 0.0234 instead of the usual 0.02.
    _fill_and_compare(wl, [230, 60], k_scale={19: 8.0, 53: 8.0, 100: 8.0, 131: 8.0, 150: 8.0, 192: 8.0, 210: 8.0, 250: 16.0},
                      out_tol=1.5 * 2.0 ** -6)


@pytest.mark.parametrize("flags", [lf.LF_FLAG_FORCE_SPLIT, lf.LF_FLAG_FORCE_UNIT, lf.LF_FLAG_FORCE_VALU],
                         ids=["split", "unit", "valu"])
def test_bulk_fill_on_every_kernel_path(flags):
    wl = _wl("fill_paths", "bf16", 2, 14, 2, 128, 600, n_init=100, sink_scale=4.0, seed=41)
    _fill_and_compare(wl, [250, 250], flags=flags)


@pytest.mark.parametrize("dtype,D", [("f32", 64), ("f32", 128), ("bf16", 64)])
def test_bulk_fill_of_caches_without_the_batched_kernel_runs_the_steps(dtype, D):
    wl = _wl(f"fill_{dtype}_d{D}", dtype, 2, 8, 2, D, 90, n_init=5, seed=3)
    _fill_and_compare(wl, [40, 45])


def test_bulk_fill_equals_sequential_steps_on_the_gpu():
    wl = _wl("fill_vs_steps", "bf16", 4, 28, 4, 128, 400, n_init=10, seed=8)
    k0, v0 = W.device_prefill(wl, "cuda")
    a = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, 128, wl.budget, k_init=k0, v_init=v0)
    b = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, 128, wl.budget, k_init=k0, v_init=v0)
    T = wl.budget - wl.n_init
    q, k, v = _stack_steps(wl, 0, T)
    out_a, idx_a = a.fill_steps(q, k, v)
    outs = []
    for t in range(T):
        o, idx_b = b.decode_step(q[t], k[t], v[t])
        outs.append(o.clone())
    torch.cuda.synchronize()
    out_b = torch.stack(outs)
    assert torch.equal(idx_a, idx_b)                       # the eviction decision of the step that filled the cache
    assert torch.equal(a.k_cache.view(torch.int16), b.k_cache.view(torch.int16))
    assert torch.equal(a.v_cache.view(torch.int16), b.v_cache.view(torch.int16))
    # same sums in another order: a bf16 ulp of |out| <= 4 at most
    assert (out_a.float() - out_b.float()).abs().max().item() <= 2 ** -6
    assert torch.equal(out_a[-1].view(torch.int16), out_b[-1].view(torch.int16))   # the last token took the same kernel
    sa, sb = a.scores(), b.scores()
    assert torch.equal(sa, sb)


def test_cfg3_geometry_bulk_fill_to_the_brim_sampled_units():
    wl = W.scaled(W.CONFIGS[3], name="cfg3_fill", layers=1, n_init=W.CONFIGS[3].budget - 96)
    rng = np.random.default_rng(11)
    units = np.sort(rng.choice(wl.units, size=12, replace=False))
    rep, gpu, _ = _fill_and_compare(wl, [96], units=units, tail_steps=2)
    print(f"\ncfg3 fill: decisions {rep.decisions} near-ties {rep.near_ties} max|dout| {rep.max_out_err:.2e}")
    gpu.close()
    del gpu
    torch.cuda.empty_cache()


@pytest.mark.parametrize("Hq,Hkv,N,n_init,chunks,flags", [
    (28, 4, 300, 100, [150, 120, 40], 0),                   # second chunk crosses the brim, third only evicts
    (8, 2, 200, 0, [450], 0),                               # a "prompt" of 450 tokens into 200 slots in one call
    (14, 2, 700, 690, [5, 30], lf.LF_FLAG_FORCE_SPLIT),     # too few free slots for the batched kernel
], ids=lambda v: str(v).replace(" ", ""))
def test_tokens_beyond_the_free_slots_evict_as_single_steps_do(Hq, Hkv, N, n_init, chunks, flags):
    wl = _wl(f"over_{Hq}x{Hkv}_n{N}", "bf16", 2, Hq, Hkv, 128, N, n_init=n_init, sink_scale=4.0, seed=700 + N)
    rep, gpu, ora = _fill_and_compare(wl, chunks, flags=flags, tail_steps=5)
    assert gpu.valid_count == N


def test_multi_token_call_on_a_masked_cache_runs_the_steps():
    wl = _wl("fill_masked", "bf16", 2, 14, 2, 128, 400, n_init=400, seed=77)
    k0, v0 = W.device_prefill(wl, "cuda")
    gpu = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, 128, wl.budget, k_init=k0, v_init=v0)
    ora = oracle.OracleCache(wl.units, wl.group, 1, 128, wl.budget)
    ora.init(W.to_f64(k0.reshape(wl.units, 1, 400, 128)), W.to_f64(v0.reshape(wl.units, 1, 400, 128)))
    mask = np.random.default_rng(4).random((wl.units, 400)) < 0.9
    mask[:, 0] = True
    gpu.set_pending(torch.zeros((wl.batch, wl.kv_heads), dtype=torch.int32))
    ora.set_pending(np.zeros((wl.units, 1), dtype=np.int32))
    gpu.set_mask(torch.as_tensor(mask.reshape(wl.batch, wl.kv_heads, 400)))
    ora.set_mask(mask.reshape(wl.units, 1, 400))
    T = 60                                                   # ~40 holes per unit get filled, then eviction
    q, k, v = _stack_steps(wl, 0, T)
    out_t, idx_t = gpu.fill_steps(q, k, v)
    torch.cuda.synchronize()
    o_ref, i_ref = ora.fill(W.to_f64(q.reshape(T, wl.units, wl.group, 128)), W.to_f64(k.reshape(T, wl.units, 1, 128)),
                            W.to_f64(v.reshape(T, wl.units, 1, 128)))
    assert np.abs(W.to_f64(out_t.reshape(T, wl.units, wl.group, 128)) - o_ref).max() <= OUT_TOL["bf16"]
    assert (idx_t.reshape(-1).cpu().numpy() == i_ref.reshape(-1)).all()
    assert (gpu.mask().reshape(wl.units, 400).cpu().numpy() == ora.mask().reshape(wl.units, 400)).all()


def test_bulk_fill_argument_errors():
    c = lf.LongFlowCache(1, 4, 1, 128, 64)
    q = torch.zeros(65, 1, 4, 128, device="cuda", dtype=torch.bfloat16)
    kv = torch.zeros(65, 1, 1, 128, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(lf.LongFlowError):
        c.fill_steps(q[:0], kv[:0], kv[:0])                  # no token
    c.fill_steps(q, kv, kv)                                  # 65 tokens into 64 slots: the last one evicts
    assert c.valid_count == 64
    born_full = lf.LongFlowCache(1, 4, 1, 128, 64, k_init=kv[:64].reshape(1, 1, 64, 128), v_init=kv[:64].reshape(1, 1, 64, 128))
    with pytest.raises(lf.LongFlowError):
        born_full.fill_steps(q[:2], kv[:2], kv[:2])          # full and no slot named yet
    ao = lf.LongFlowCache(1, 4, 1, 128, 64, flags=lf.LF_FLAG_ATTENTION_ONLY, k_init=kv[:8].reshape(1, 1, 8, 128),
                          v_init=kv[:8].reshape(1, 1, 8, 128))
    with pytest.raises(lf.LongFlowError):
        ao.fill_steps(q[:1], kv[:1], kv[:1])
    torch.cuda.synchronize()


def test_bulk_fill_of_degenerate_budgets():
    for N in (1, 2, 3, 15, 16, 17):
        wl = _wl(f"fill_tiny_{N}", "bf16", 2, 2, 2, 128, N, seed=300 + N)       # G = 1: 64 tokens per pass
        _fill_and_compare(wl, [N], tail_steps=4)
        if N > 2:
            _fill_and_compare(wl, [1, N - 2, 1], tail_steps=2)
