"""GPU parity: the HIP decode path, called through the C ABI, against the float64 oracle."""
import numpy as np
import pytest
import torch

from oracle import longflow_oracle as oracle
from paper_2603_11504_amd import longflow as lf
from paper_2603_11504_amd import workloads as W

from parity import OUT_TOL, ParityReport, compare_indices, run_lockstep

pytestmark = pytest.mark.gpu


def _small(name, dtype, B, Hq, Hkv, D, N, n_init=0, steps=0, **kw):
    return W.Workload(name, dtype, B, Hq, Hkv, D, N, n_init, steps or 2 * N, **kw)


# ------------------------------------------------------------------ BASELINE configs 0 and 1, every step

def test_cfg0_fp32_every_step_with_scores():
    wl = W.CONFIGS[0]
    rep, _, _ = run_lockstep(wl, check_scores_every=16)
    print(f"\ncfg0: steps {rep.steps} decisions {rep.decisions} near-ties {rep.near_ties} "
          f"max|dout| {rep.max_out_err:.2e} max score rel {rep.max_score_rel:.2e}")
    assert rep.steps == 512


@pytest.mark.parametrize("flags", [0, lf.LF_FLAG_FORCE_VALU], ids=["default", "valu"])
def test_cfg1_bf16_every_step(flags):
    wl = W.CONFIGS[1]
    rep, _, _ = run_lockstep(wl, flags=flags, check_scores_every=512)
    print(f"\ncfg1[{flags}]: steps {rep.steps} decisions {rep.decisions} near-ties {rep.near_ties} "
          f"max|dout| {rep.max_out_err:.2e} max score rel {rep.max_score_rel:.2e}")
    assert rep.steps == 4096


# ------------------------------------------------------------------ shapes: groups, head dims, ragged budgets

@pytest.mark.parametrize("dtype,Hq,Hkv,D,N,flags", [
    ("f32", 1, 1, 64, 37, 0), ("f32", 6, 2, 128, 100, 0), ("f32", 8, 1, 64, 333, 0),
    ("bf16", 2, 2, 64, 50, 0), ("bf16", 3, 1, 64, 272, 0), ("bf16", 10, 2, 128, 129, 0),
    # groups beyond 8 heads on the fp32 matrix-core kernel; its vector-ALU twin
    ("f32", 16, 1, 64, 300, 0), ("f32", 26, 2, 128, 530, 0), ("bf16", 12, 1, 64, 700, 0), ("f32", 7, 1, 128, 1100, 0),
    ("f32", 6, 2, 128, 100, lf.LF_FLAG_FORCE_VALU), ("f32", 8, 1, 64, 333, lf.LF_FLAG_FORCE_VALU),
    ("bf16", 3, 1, 64, 272, lf.LF_FLAG_FORCE_VALU),
    ("bf16", 7, 1, 128, 1000, 0), ("bf16", 8, 1, 128, 515, lf.LF_FLAG_FORCE_VALU),
    ("bf16", 16, 1, 128, 300, 0), ("bf16", 24, 2, 128, 2100, 0),
    # one fused launch per step, one workgroup per unit
    ("bf16", 1, 1, 128, 61, lf.LF_FLAG_FORCE_UNIT), ("bf16", 14, 2, 128, 129, lf.LF_FLAG_FORCE_UNIT),
    ("bf16", 7, 1, 128, 1000, lf.LF_FLAG_FORCE_UNIT), ("bf16", 16, 1, 128, 300, lf.LF_FLAG_FORCE_UNIT),
    ("bf16", 10, 2, 128, 2100, lf.LF_FLAG_FORCE_UNIT),
])
def test_shapes_fill_then_evict(dtype, Hq, Hkv, D, N, flags):
    wl = _small(f"shape_{dtype}_{Hq}x{Hkv}_d{D}_n{N}", dtype, 3, Hq, Hkv, D, N, steps=N + 40,
                sink_scale=4.0, seed=77 + N)
    rep, _, _ = run_lockstep(wl, flags=flags, check_scores_every=97)
    assert rep.steps == N + 40


@pytest.mark.parametrize("flags", [lf.LF_FLAG_FORCE_SPLIT, lf.LF_FLAG_FORCE_UNIT], ids=["split", "unit"])
def test_prefilled_caches_of_every_fill_level(flags):
    # n_init from nearly empty to one short of full, ragged against tiles and splits
    for n_init in (1, 15, 16, 17, 127, 128, 129, 255, 256, 257, 599):
        wl = _small(f"prefill_{n_init}", "bf16", 2, 14, 2, 128, 600, n_init=n_init, steps=12, seed=5 + n_init)
        run_lockstep(wl, flags=flags, check_scores_every=5)


# ------------------------------------------------------------------ larger configs at full size, sampled units

@pytest.mark.parametrize("flags", [0, lf.LF_FLAG_FORCE_UNIT], ids=["default", "unit"])
def test_cfg2_full_size_all_units(flags):
    wl = W.CONFIGS[2]
    rep, gpu, _ = run_lockstep(wl, steps=4, flags=flags, host_inputs=False, check_scores_every=3)
    print(f"\ncfg2[{flags}]: decisions {rep.decisions} near-ties {rep.near_ties} max|dout| {rep.max_out_err:.2e}")
    gpu.close()


def test_cfg3_one_layer_split_path():
    wl = W.CONFIGS[3]
    units = np.arange(0, wl.units, 8)
    rep, gpu, _ = run_lockstep(wl, steps=2, flags=lf.LF_FLAG_FORCE_SPLIT, host_inputs=False, units=units, layer=3)
    print(f"\ncfg3 split path: decisions {rep.decisions} near-ties {rep.near_ties} max|dout| {rep.max_out_err:.2e}")
    gpu.close()
    del gpu
    torch.cuda.empty_cache()


def test_cfg3_full_size_sampled_units_two_layers():
    wl = W.CONFIGS[3]
    rng = np.random.default_rng(wl.seed)
    for layer in (0, 27):
        units = np.sort(rng.choice(wl.units, size=64, replace=False))
        rep, gpu, _ = run_lockstep(wl, steps=4, host_inputs=False, units=units, layer=layer)
        print(f"\ncfg3 layer {layer}: decisions {rep.decisions} near-ties {rep.near_ties} max|dout| {rep.max_out_err:.2e}")
        gpu.close()
        del gpu
        torch.cuda.empty_cache()


def test_cfg4_full_size_sampled_units():
    wl = W.CONFIGS[4]
    rng = np.random.default_rng(wl.seed)
    units = np.sort(rng.choice(wl.units, size=64, replace=False))
    rep, gpu, _ = run_lockstep(wl, steps=3, host_inputs=False, units=units)
    print(f"\ncfg4: decisions {rep.decisions} near-ties {rep.near_ties} max|dout| {rep.max_out_err:.2e}")
    gpu.close()
    del gpu
    torch.cuda.empty_cache()


@pytest.mark.parametrize("B,Hq,Hkv,N,sample", [
    (48, 8, 4, 20000, 8),    # one workgroup per unit, more slots than its register window screens in one pass
    (1, 8, 2, 60000, None),  # eight workgroups per unit, their codes copied a chunk at a time, decoded twice
    (1, 32, 2, 16000, None), # the same with 16 heads a group inside the register window: chunks, one decode pass
    (1, 7, 1, 200000, None), # codes exceed LDS even eight ways: the split-K path is chosen by itself
    (1, 2, 1, 1 << 24, None), # the largest budget the interface accepts (4 GiB of K, 4 GiB of V in one unit)
])
def test_long_budgets(B, Hq, Hkv, N, sample):
    wl = _small(f"long_{N}", "bf16", B, Hq, Hkv, 128, N, n_init=N - 2, steps=5, sink_scale=4.0, seed=N)
    units = None if sample is None else np.arange(0, wl.units, wl.units // sample)
    rep, gpu, _ = run_lockstep(wl, host_inputs=False, units=units, check_scores_every=4)
    print(f"\nlong budget {N}: decisions {rep.decisions} near-ties {rep.near_ties} max|dout| {rep.max_out_err:.2e}")
    assert rep.steps == 5
    gpu.close()
    del gpu
    torch.cuda.empty_cache()


@pytest.mark.parametrize("flags", [0, lf.LF_FLAG_FORCE_SPLIT], ids=["unit", "split"])
def test_largest_unit_count_the_interface_accepts(flags):
    # 2^20 (batch, KV head) units of 16 slots: one workgroup each, 4 GiB of K and of V
    wl = _small("max_units", "bf16", 131072, 8, 8, 128, 16, n_init=13, steps=8, sink_scale=4.0, seed=5)
    units = np.unique(np.concatenate([[0, wl.units - 1], np.random.default_rng(1).choice(wl.units, 200)]))
    rep, gpu, _ = run_lockstep(wl, host_inputs=False, check_scores_every=7, units=units, flags=flags)
    assert rep.steps == 8
    gpu.close()
    del gpu
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ edge cases

@pytest.mark.parametrize("dtype,D,flags", [("f32", 64, 0), ("f32", 128, 0), ("bf16", 64, 0), ("bf16", 128, lf.LF_FLAG_FORCE_UNIT),
                                           ("bf16", 128, lf.LF_FLAG_FORCE_SPLIT), ("bf16", 128, lf.LF_FLAG_FORCE_VALU)],
                         ids=["f32-64", "f32-128", "bf16-64", "unit", "split", "valu"])
def test_degenerate_budgets_of_a_few_slots(dtype, D, flags):
    # N = 1: every token replaces the only slot and attention returns its own value row;
    # N = 2, 3: the argmin runs over a handful of slots; 15, 16, 17: around one tile
    for N in (1, 2, 3, 15, 16, 17):
        wl = _small(f"tiny_{N}", dtype, 2, 6, 2, D, N, steps=N + 12, sink_scale=4.0, seed=300 + N)
        rep, gpu, ora = run_lockstep(wl, flags=flags, check_scores_every=1)
        assert rep.steps == N + 12
        if N == 1:
            assert (gpu.evict_idx.cpu().numpy() == 0).all()



@pytest.mark.parametrize("flags", [lf.LF_FLAG_FORCE_SPLIT, lf.LF_FLAG_FORCE_UNIT], ids=["split", "unit"])
def test_deterministic_bitwise(flags):
    wl = _small("det", "bf16", 4, 28, 4, 128, 700, n_init=699, steps=20, seed=11)
    runs = []
    for _ in range(2):
        k0, v0 = W.host_prefill(wl)
        gpu = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, flags=flags,
                               k_init=W.to_torch(k0, wl, "cuda"), v_init=W.to_torch(v0, wl, "cuda"))
        outs, idxs = [], []
        for t in range(wl.steps):
            q, k, v = (W.to_torch(x, wl, "cuda") for x in W.host_step(wl, t))
            o, i = gpu.decode_step(q, k, v)
            outs.append(o.clone()); idxs.append(i.clone())
        torch.cuda.synchronize()
        runs.append((torch.stack(outs), torch.stack(idxs)))
    assert torch.equal(runs[0][0].view(torch.int16), runs[1][0].view(torch.int16))
    assert torch.equal(runs[0][1], runs[1][1])


@pytest.mark.parametrize("flags", [lf.LF_FLAG_FORCE_SPLIT, lf.LF_FLAG_FORCE_UNIT], ids=["split", "unit"])
def test_insert_lands_in_named_slot_at_tile_and_split_edges(flags):
    wl = _small("edges", "bf16", 2, 7, 1, 128, 2048 + 256, n_init=2048 + 255, steps=1, seed=21)
    rep, gpu, ora = run_lockstep(wl, steps=1, flags=flags)
    N = wl.budget
    for t, slot in enumerate([0, 15, 16, 255, 256, 1023, 1024, 2047, 2048, N - 1], start=1):
        pend = np.full((wl.units, 1), slot, dtype=np.int32)
        gpu.set_pending(torch.from_numpy(pend.reshape(wl.batch, wl.kv_heads)))
        ora.set_pending(pend)
        q, k, v = (W.to_torch(x, wl, "cuda") for x in W.host_step(wl, t))
        out, idx = gpu.decode_step(q, k, v)
        torch.cuda.synchronize()
        assert torch.equal(gpu.k_cache[:, :, slot, :], k) and torch.equal(gpu.v_cache[:, :, slot, :], v)
        o_ref, i_ref = ora.step(W.to_f64(q).reshape(wl.units, wl.group, -1), W.to_f64(k).reshape(wl.units, 1, -1),
                                W.to_f64(v).reshape(wl.units, 1, -1))
        assert np.abs(W.to_f64(out).reshape(o_ref.shape) - o_ref).max() <= 2e-2
        compare_indices(idx.cpu().numpy(), i_ref, ora.scores(), True, rep, where=f"slot {slot}")
        Kc, _ = ora.kv()
        np.testing.assert_array_equal(W.to_f64(gpu.k_cache).reshape(Kc.shape), Kc)


@pytest.mark.parametrize("flags", [0, lf.LF_FLAG_FORCE_UNIT, lf.LF_FLAG_FORCE_SPLIT], ids=["default", "unit", "split"])
def test_a_dominant_new_token_is_attended_in_whatever_tile_it_lands(flags):
    # The heads of a group share one query, the new token's key is that query scaled up, its value is a
    # constant: the output must be that constant.  A kernel that streamed the slot's old row (say from a
    # tile it had requested before the insert) would return the cache's average instead.  The slots lie in
    # a wave's first, second and third tile, just behind them, and at the ends.
    wl = _small("dominant", "bf16", 3, 14, 2, 128, 1024, n_init=1023, steps=1, seed=41)
    rep, gpu, ora = run_lockstep(wl, steps=1, flags=flags)
    G, D = wl.group, 128
    def put(slot, t, dominant):
        pend = np.full((wl.units, 1), slot, dtype=np.int32)
        gpu.set_pending(torch.from_numpy(pend.reshape(wl.batch, wl.kv_heads)))
        ora.set_pending(pend)
        q, k, v = W.host_step(wl, t)
        if dominant:
            q = np.repeat(q.reshape(wl.batch, wl.kv_heads, G, D)[:, :, :1], G, axis=2).reshape(q.shape)
            k = W.round_to_storage(4.0 * q.reshape(wl.batch, wl.kv_heads, G, D)[:, :, 0], "bf16").reshape(k.shape)
            v = np.full_like(v, 3.0)
        return q, k, v

    prev = None
    for t, slot in enumerate([5, 16 * 8 + 3, 16 * 9 + 1, 16 * 23 + 15, 16 * 24, 16 * 30 + 7, 0, 1023], start=1):
        if prev is not None:   # an ordinary token takes the last dominant one's place first
            q, k, v = put(prev, 100 + t, False)
            gpu.decode_step(*(W.to_torch(x, wl, "cuda") for x in (q, k, v)))
            ora.step(q.astype(np.float64).reshape(wl.units, G, D), k.astype(np.float64).reshape(wl.units, 1, D),
                     v.astype(np.float64).reshape(wl.units, 1, D))
        prev = slot
        q, k, v = put(slot, t, True)
        out, idx = gpu.decode_step(*(W.to_torch(x, wl, "cuda") for x in (q, k, v)))
        torch.cuda.synchronize()
        o_ref, i_ref = ora.step(q.astype(np.float64).reshape(wl.units, G, D), k.astype(np.float64).reshape(wl.units, 1, D),
                                v.astype(np.float64).reshape(wl.units, 1, D))
        o_gpu = W.to_f64(out).reshape(o_ref.shape)
        assert np.abs(o_ref - 3.0).max() < 0.3                       # the construction works: the new token takes the weight
        assert np.abs(o_gpu - o_ref).max() <= 2e-2, f"slot {slot}"
        compare_indices(idx.cpu().numpy(), i_ref, ora.scores(), True, rep, where=f"slot {slot}")
    gpu.close()


@pytest.mark.parametrize("flags", [lf.LF_FLAG_FORCE_SPLIT, lf.LF_FLAG_FORCE_UNIT], ids=["split", "unit"])
def test_exact_ties_evict_the_lowest_index(flags):
    # two bit-identical rows that are jointly the least important: the tie is exact in
    # the oracle, and the screening + exact re-scoring must resolve it to the lower slot
    wl = _small("ties", "bf16", 1, 7, 1, 128, 512, n_init=511, steps=1, seed=31)
    k0, v0 = W.host_prefill(wl)
    q, k, v = W.host_step(wl, 0)
    low_k = W.round_to_storage(-0.5 * q.sum(1, keepdims=True), "bf16")   # every head's logit far below the rest
    low_v = W.round_to_storage(np.full((1, 1, 128), 2.0 ** -6, np.float32), "bf16")
    for s in (300, 77, 450):
        k0[:, :, s] = low_k
        v0[:, :, s] = low_v
    gpu = lf.LongFlowCache(1, 7, 1, 128, 512, flags=flags, k_init=W.to_torch(k0, wl, "cuda"),
                           v_init=W.to_torch(v0, wl, "cuda"))
    ora = oracle.OracleCache(1, 7, 1, 128, 512)
    ora.init(k0.astype(np.float64), v0.astype(np.float64))
    _, idx = gpu.decode_step(*(W.to_torch(x, wl, "cuda") for x in (q, k, v)))
    _, i_ref = ora.step(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64))
    sc = ora.scores()[0, 0]
    assert sc[77] == sc[300] == sc[450] == sc.min()       # the construction worked
    assert int(i_ref[0, 0]) == 77
    assert int(idx.cpu()[0, 0]) == 77


@pytest.mark.parametrize("D,flags", [(64, 0), (128, lf.LF_FLAG_FORCE_SPLIT), (128, lf.LF_FLAG_FORCE_UNIT)],
                         ids=["valu", "split", "unit"])
def test_wide_logit_range_underflow_is_resolved_exactly(D, flags):
    # logits spread over hundreds of nats: most fp32 probabilities underflow to zero, the
    # screening sees many zeros, and the exact re-scoring must still find the oracle's slot
    wl = _small("underflow", "bf16", 2, 4, 2, D, 256, n_init=255, steps=6, seed=41,
                channel_scale_range=(20.0, 40.0))
    rep, _, _ = run_lockstep(wl, steps=6, flags=flags)
    assert rep.near_ties == 0


@pytest.mark.parametrize("flags", [lf.LF_FLAG_FORCE_SPLIT, lf.LF_FLAG_FORCE_UNIT], ids=["split", "unit"])
def test_attention_only_flag_leaves_cache_untouched(flags):
    wl = _small("attn_only", "bf16", 2, 10, 2, 128, 1500, n_init=1500, steps=1, seed=51)
    k0, v0 = W.host_prefill(wl)
    gpu = lf.LongFlowCache(2, 10, 2, 128, 1500, flags=lf.LF_FLAG_ATTENTION_ONLY | flags,
                           k_init=W.to_torch(k0, wl, "cuda"), v_init=W.to_torch(v0, wl, "cuda"))
    before = gpu.k_cache.clone()
    q, _, _ = W.host_step(wl, 0)
    out, _ = gpu.decode_step(W.to_torch(q, wl, "cuda"))
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.int16), gpu.k_cache.view(torch.int16))
    for u in range(4):
        o_ref, _, _ = oracle.attend_unit(q.reshape(4, 5, 128)[u], k0.reshape(4, 1500, 128)[u], v0.reshape(4, 1500, 128)[u])
        assert np.abs(W.to_f64(out).reshape(4, 5, 128)[u] - o_ref).max() <= 2e-2
    with pytest.raises(lf.LongFlowError):
        gpu.scores()


def test_full_cache_needs_a_pending_slot():
    wl = _small("born_full", "f32", 1, 4, 1, 64, 64, n_init=64, steps=1, seed=61)
    k0, v0 = W.host_prefill(wl)
    gpu = lf.LongFlowCache(1, 4, 1, 64, 64, dtype=torch.float32, k_init=W.to_torch(k0, wl, "cuda"),
                           v_init=W.to_torch(v0, wl, "cuda"))
    q, k, v = (W.to_torch(x, wl, "cuda") for x in W.host_step(wl, 0))
    with pytest.raises(lf.LongFlowError) as e:
        gpu.decode_step(q, k, v)
    assert e.value.status == lf.LF_ERR_STATE
    with pytest.raises(lf.LongFlowError):
        gpu.scores()
    gpu.set_pending(torch.tensor([[9]], dtype=torch.int32))
    gpu.decode_step(q, k, v)
    torch.cuda.synchronize()
    assert torch.equal(gpu.k_cache[0, 0, 9], k[0, 0])


# ------------------------------------------------------------------ HIP graph capture

@pytest.mark.parametrize("flags", [lf.LF_FLAG_FORCE_SPLIT, lf.LF_FLAG_FORCE_UNIT], ids=["split", "unit"])
def test_decode_steps_replayed_from_a_hip_graph_match_eager(flags):
    # a full cache advances by pure kernel launches (no allocation, no memset, no host sync), so a
    # caller may capture steady-state steps in a HIP graph; every replay must equal the eager path
    wl = _small("graph", "bf16", 4, 28, 4, 128, 1024, n_init=1023, steps=8, seed=71)
    k0, v0 = W.host_prefill(wl)
    mk = lambda: lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, flags=flags,
                                  k_init=W.to_torch(k0, wl, "cuda"), v_init=W.to_torch(v0, wl, "cuda"))
    eager, graphed = mk(), mk()
    qs, ks, vs = (torch.empty_like(W.to_torch(x, wl, "cuda")) for x in W.host_step(wl, 0))
    for t in range(2):                                   # fill completes, kernels are loaded
        for dst, src in zip((qs, ks, vs), W.host_step(wl, t)):
            dst.copy_(W.to_torch(src, wl, "cuda"))
        eager.decode_step(qs, ks, vs)
        graphed.decode_step(qs, ks, vs)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.decode_step(qs, ks, vs)
    # capturing does not execute: eager has to catch up with nothing
    for t in range(2, 8):
        for dst, src in zip((qs, ks, vs), W.host_step(wl, t)):
            dst.copy_(W.to_torch(src, wl, "cuda"))
        o_e, i_e = eager.decode_step(qs, ks, vs)
        o_e, i_e = o_e.clone(), i_e.clone()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_e.view(torch.int16), graphed.out.view(torch.int16)), f"replay {t}"
        assert torch.equal(i_e, graphed.evict_idx), f"replay {t}"
        junk = torch.randn(1 << 20, device="cuda").sum().item()   # unrelated eager work between replays
        assert junk == junk
    assert torch.equal(eager.k_cache.view(torch.int16), graphed.k_cache.view(torch.int16))


def test_grouped_masked_steps_replayed_from_a_hip_graph_match_eager():
    # one captured launch serving three caches that carry an explicit mask with a few holes:
    # the replays fill the holes and go on evicting exactly as the eager calls do
    wl = _small("graph-group", "bf16", 2, 16, 4, 128, 768, n_init=768, steps=1, seed=72)
    mask = _random_mask(wl, 3, 0.995)
    sets = []
    for _ in range(2):
        caches = _make_caches(wl, 3)
        for c in caches:
            c.set_pending(torch.zeros((wl.batch, wl.kv_heads), dtype=torch.int32))
            c.set_mask(torch.as_tensor(mask))
        sets.append((caches, lf.LongFlowGroup(caches)))
    (ce, ge), (cg, gg) = sets
    qs, ks, vs = (torch.stack([W.to_torch(x, wl, "cuda")] * 3) for x in W.host_step(wl, 0))

    def load(t):
        for j in range(3):
            for dst, src in zip((qs, ks, vs), W.host_step(wl, t, j)):
                dst[j].copy_(W.to_torch(src, wl, "cuda"))

    load(0)
    ge.decode_step(qs, ks, vs)
    gg.decode_step(qs, ks, vs)                            # kernels loaded before the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        gg.decode_step(qs, ks, vs)
    for t in range(1, 14):
        load(t)
        o_e, i_e = ge.decode_step(qs, ks, vs)
        o_e, i_e = o_e.clone(), i_e.clone()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_e.view(torch.int16), gg.out.view(torch.int16)), f"replay {t}"
        assert torch.equal(i_e, gg.evict_idx), f"replay {t}"
        assert torch.randn(1 << 18, device="cuda").sum().item() is not None   # unrelated eager work between replays
    for a_, b_ in zip(ce, cg):
        assert torch.equal(a_.mask(), b_.mask()) and bool(a_.mask().all())
    ge.close(); gg.close()
    for c in ce + cg:
        c.close()


# ------------------------------------------------------------------ newest token as eviction candidate

@pytest.mark.parametrize("flags,B", [(0, 1), (lf.LF_FLAG_FORCE_UNIT, 1), (lf.LF_FLAG_FORCE_SPLIT, 1), (0, 40)],
                         ids=["coop", "single", "split", "coop-many"])
def test_just_inserted_row_competes_for_eviction(flags, B):
    # Every new token is built to score within a few percent of a decoy row, so the exact
    # re-scoring must read the row that was written moments ago in the same launch -- with
    # several workgroups per unit, by a different workgroup than the one deciding.
    Hq, Hkv, D, N = 14, 2, 128, 2048
    wl = _small("fresh", "bf16", B, Hq, Hkv, D, N, n_init=N - 1, steps=1, seed=91)
    rng = np.random.default_rng(7)
    k0, v0 = W.host_prefill(wl)
    q = W.round_to_storage(rng.standard_normal((B, Hq, D)).astype(np.float32), "bf16")   # same query every step
    qsum = q.reshape(B, Hkv, Hq // Hkv, D).sum(2)
    low_k = W.round_to_storage(-0.5 * qsum, "bf16")                                       # every head's logit far down
    base_v = np.full((B, Hkv, D), 2.0 ** -4, np.float32)
    k0[:, :, 100] = low_k
    v0[:, :, 100] = base_v                                                                # the decoy
    gpu = lf.LongFlowCache(B, Hq, Hkv, D, N, flags=flags, k_init=W.to_torch(k0, wl, "cuda"),
                           v_init=W.to_torch(v0, wl, "cuda"))
    ora = oracle.OracleCache(B * Hkv, Hq // Hkv, 1, D, N)
    ora.init(k0.reshape(B * Hkv, 1, N - 1, D).astype(np.float64), v0.reshape(B * Hkv, 1, N - 1, D).astype(np.float64))
    rep = ParityReport()
    fresh_evicted = 0
    for t in range(16):
        scale = 1.0 + 0.03 * ((-1) ** t) * (1 + t % 3)            # a little above / below the decoy
        v_new = W.round_to_storage(base_v * np.float32(scale), "bf16")
        out, idx = gpu.decode_step(W.to_torch(q, wl, "cuda"), W.to_torch(low_k, wl, "cuda"), W.to_torch(v_new, wl, "cuda"))
        torch.cuda.synchronize()
        pend_before = ora.pending().reshape(-1).copy()
        o_ref, i_ref = ora.step(q.reshape(B * Hkv, -1, D).astype(np.float64), low_k.reshape(B * Hkv, 1, D).astype(np.float64),
                                v_new.reshape(B * Hkv, 1, D).astype(np.float64))
        assert np.abs(W.to_f64(out).reshape(o_ref.shape) - o_ref).max() <= 2e-2
        i_gpu = idx.cpu().numpy().reshape(-1)
        if compare_indices(i_gpu, i_ref, ora.scores(), True, rep, where=f"fresh step {t}"):
            ora.set_pending(i_gpu.reshape(-1, 1))
        fresh_evicted += int((i_ref.reshape(-1) == pend_before).sum())
    assert fresh_evicted > 0          # the construction does make the newest row the minimum at times


# ------------------------------------------------------------------ random geometries

def _random_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        D = 128 if rng.random() < 0.7 else 64
        mfma_ok = dtype == "bf16" and D == 128
        flags = int(rng.choice([0, 0, lf.LF_FLAG_FORCE_VALU]))
        if mfma_ok:
            flags = int(rng.choice([0, 0, lf.LF_FLAG_FORCE_SPLIT, lf.LF_FLAG_FORCE_UNIT, lf.LF_FLAG_FORCE_VALU]))
        gmax = 8 if flags & lf.LF_FLAG_FORCE_VALU else 16
        G = int(rng.integers(1, gmax + 1))
        Hkv = int(rng.integers(1, 4))
        B = int(rng.integers(1, 6))
        N = int(rng.choice([int(rng.integers(17, 200)), int(rng.integers(200, 1200)), int(rng.integers(1200, 3000))]))
        n_init = int(rng.choice([max(0, N - int(rng.integers(1, 40))), N - 1, int(rng.integers(0, N))]))
        steps = int(min(N - n_init + 12, 48))
        cases.append((dtype, B, G * Hkv, Hkv, D, N, n_init, steps, flags, int(rng.integers(1 << 30))))
    return cases


@pytest.mark.parametrize("case", _random_cases(36, 20260311), ids=lambda c: "-".join(str(x) for x in c[:9]))
def test_random_geometries(case):
    dtype, B, Hq, Hkv, D, N, n_init, steps, flags, seed = case
    wl = W.Workload("rand", dtype, B, Hq, Hkv, D, N, n_init, steps, sink_scale=4.0 if seed & 1 else 1.0,
                    outlier_channels=4 if seed & 2 else 0, outlier_scale=8.0, seed=seed)
    rep, gpu, _ = run_lockstep(wl, flags=flags, check_scores_every=7)
    assert rep.steps == steps
    gpu.close()


# ------------------------------------------------------------------ independent caches on several streams

def test_independent_caches_on_two_streams_match_serial_execution():
    # handles share no mutable state: driving them from different streams gives the same bits
    wl = _small("streams", "bf16", 8, 28, 4, 128, 1024, n_init=1023, steps=6, seed=81)
    outs = {}
    for mode in ("serial", "streams"):
        caches = []
        for layer in range(4):
            k0, v0 = W.host_prefill(wl, layer)
            caches.append(lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget,
                                           k_init=W.to_torch(k0, wl, "cuda"), v_init=W.to_torch(v0, wl, "cuda")))
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        torch.cuda.synchronize()
        res = []
        for t in range(wl.steps):
            for layer, c in enumerate(caches):
                q, k, v = (W.to_torch(x, wl, "cuda") for x in W.host_step(wl, t, layer))
                if mode == "streams":
                    streams[layer % 2].wait_stream(torch.cuda.current_stream())
                    with torch.cuda.stream(streams[layer % 2]):
                        o, i = c.decode_step(q, k, v)
                        res.append((o.clone(), i.clone()))
                else:
                    o, i = c.decode_step(q, k, v)
                    res.append((o.clone(), i.clone()))
        torch.cuda.synchronize()
        outs[mode] = res
        for c in caches:
            c.close()
    for (o1, i1), (o2, i2) in zip(outs["serial"], outs["streams"]):
        assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)) and torch.equal(i1, i2)


# ------------------------------------------------------------------ several caches in one launch

class _GroupMember:
    """Looks like one LongFlowCache to run_lockstep; every step runs the whole group."""

    def __init__(self, group, j, wl, seed):
        self.group, self.j, self.wl = group, j, wl
        self.gen = torch.Generator(device="cuda").manual_seed(seed)

    def decode_step(self, q, k, v):
        n = len(self.group.caches)
        dt = W.torch_dtype(self.wl)
        qa = torch.randn((n,) + tuple(q.shape), device="cuda", dtype=torch.float32, generator=self.gen).to(dt)
        ka = torch.randn((n,) + tuple(k.shape), device="cuda", dtype=torch.float32, generator=self.gen).to(dt)
        va = torch.randn((n,) + tuple(v.shape), device="cuda", dtype=torch.float32, generator=self.gen).to(dt)
        qa[self.j], ka[self.j], va[self.j] = q, k, v
        out, idx = self.group.decode_step(qa, ka, va)
        return out[self.j], idx[self.j]

    @property
    def valid_count(self):
        return self.group.caches[self.j].valid_count

    def scores(self):
        return self.group.caches[self.j].scores()


def _make_caches(wl, n, flags=0):
    dt = W.torch_dtype(wl)
    caches = []
    for layer in range(n):
        k0, v0 = W.host_prefill(wl, layer)
        caches.append(lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, dtype=dt, flags=flags,
                                       k_init=None if k0 is None else W.to_torch(k0, wl, "cuda"),
                                       v_init=None if v0 is None else W.to_torch(v0, wl, "cuda")))
    return caches


@pytest.mark.parametrize("name,dtype,B,Hq,Hkv,D,N,flags", [
    ("coop", "bf16", 2, 28, 4, 128, 2048, 0),            # several workgroups per unit
    ("single", "bf16", 48, 32, 8, 128, 300, 0),           # one workgroup per unit, ragged tail
    ("split", "bf16", 4, 8, 2, 128, 1024, lf.LF_FLAG_FORCE_SPLIT),      # split-K, last arriver finishes
    ("split-big", "bf16", 40, 8, 2, 128, 2048, lf.LF_FLAG_FORCE_SPLIT), # split-K, separate (grouped) finish launch
    ("fp32", "f32", 2, 8, 2, 64, 200, 0),
    ("fp32-big", "f32", 24, 6, 2, 128, 1500, 0),
])
def test_group_step_equals_member_steps(name, dtype, B, Hq, Hkv, D, N, flags):
    # fill phase into eviction phase; the group must give every member the bits it gets alone
    wl = _small("group-" + name, dtype, B, Hq, Hkv, D, N, n_init=N - 3, steps=8, seed=91)
    alone, members = _make_caches(wl, 3, flags), _make_caches(wl, 3, flags)
    group = lf.LongFlowGroup(members)
    view = torch.int16 if dtype == "bf16" else torch.int32
    for t in range(wl.steps):
        qs, ks, vs = zip(*[[W.to_torch(x, wl, "cuda") for x in W.host_step(wl, t, layer)] for layer in range(3)])
        out, idx = group.decode_step(torch.stack(qs), torch.stack(ks), torch.stack(vs))
        for j, c in enumerate(alone):
            o1, i1 = c.decode_step(qs[j], ks[j], vs[j])
            assert torch.equal(o1.view(view), out[j].view(view)), f"{name} step {t} member {j}: out differs"
            assert torch.equal(i1, idx[j]), f"{name} step {t} member {j}: eviction index differs"
            assert members[j].valid_count == c.valid_count
    torch.cuda.synchronize()
    group.close()
    for c in alone + members:
        c.close()


@pytest.mark.parametrize("B,Hq,Hkv,N", [
    (2, 28, 4, 640),     # few units: the group keeps the cooperating workgroups
    (16, 16, 4, 1024),   # 64 units take 2 workgroups each alone, 1 each in a group of 3
])
def test_group_member_against_oracle(B, Hq, Hkv, N):
    wl = _small(f"group-oracle-{B}", "bf16", B, Hq, Hkv, 128, N, n_init=N - 40, steps=120, seed=92)
    members = _make_caches(wl, 3)
    # run_lockstep prefills its oracle from layer 0: follow member 0, the others carry noise
    group = lf.LongFlowGroup(members)
    rep, _, _ = run_lockstep(wl, gpu_cache=_GroupMember(group, 0, wl, seed=5), check_scores_every=40,
                             units=None if wl.units <= 16 else list(range(0, wl.units, 5)))
    assert rep.steps == 120 and rep.decisions > 0
    group.close()
    for c in members:
        c.close()


def test_cfg3_grouped_full_size_sampled_units():
    # the grouped launch at the benchmark's geometry: three full-size layer caches in one grid,
    # one of them followed by the oracle on sampled units
    wl = W.CONFIGS[3]
    members = []
    for layer in range(3):
        k0, v0 = W.device_prefill(wl, "cuda", layer)
        members.append(lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, k_init=k0, v_init=v0))
        del k0, v0
    group = lf.LongFlowGroup(members)
    rng = np.random.default_rng(wl.seed + 1)
    units = np.sort(rng.choice(wl.units, size=48, replace=False))
    # run_lockstep prefills its oracle from `layer`: follow that member
    rep, _, _ = run_lockstep(wl, steps=3, host_inputs=False, units=units, layer=1,
                             gpu_cache=_GroupMember(group, 1, wl, seed=6))
    print(f"\ncfg3 grouped: decisions {rep.decisions} near-ties {rep.near_ties} max|dout| {rep.max_out_err:.2e}")
    assert rep.steps == 3
    group.close()
    for c in members:
        c.close()
    del members, group
    torch.cuda.empty_cache()


def test_group_attention_only_and_errors():
    wl = _small("group-att", "bf16", 4, 16, 4, 128, 512, n_init=512, steps=2, seed=93)
    att = _make_caches(wl, 2, lf.LF_FLAG_ATTENTION_ONLY)
    twin = _make_caches(wl, 2, lf.LF_FLAG_ATTENTION_ONLY)
    g = lf.LongFlowGroup(att)
    qs = [W.to_torch(W.host_step(wl, 0, layer)[0], wl, "cuda") for layer in range(2)]
    out, _ = g.decode_step(torch.stack(qs))
    for j in range(2):
        o1, _ = twin[j].decode_step(qs[j])
        assert torch.equal(o1.view(torch.int16), out[j].view(torch.int16))
    # a member cannot be destroyed under a live group
    assert lf.lib().longflow_destroy_cache(att[0]._h) == lf.LF_ERR_STATE
    g.close()
    # members that differ in configuration or in fill level are refused
    other = _make_caches(_small("group-att2", "bf16", 4, 16, 4, 128, 256, n_init=256, steps=2, seed=94), 1,
                         lf.LF_FLAG_ATTENTION_ONLY)
    with pytest.raises(lf.LongFlowError) as e:
        lf.LongFlowGroup([att[0], other[0]])
    assert e.value.status == lf.LF_ERR_INVALID_ARG
    with pytest.raises(lf.LongFlowError) as e:
        lf.LongFlowGroup([att[0], att[0]])
    assert e.value.status == lf.LF_ERR_INVALID_ARG
    wl2 = _small("group-fill", "bf16", 4, 16, 4, 128, 512, n_init=100, steps=2, seed=95)
    fill = _make_caches(wl2, 2)
    g2 = lf.LongFlowGroup(fill)
    q, k, v = (W.to_torch(x, wl2, "cuda") for x in W.host_step(wl2, 0, 0))
    fill[0].decode_step(q, k, v)  # member 0 runs ahead
    with pytest.raises(lf.LongFlowError) as e:
        g2.decode_step(torch.stack([q, q]), torch.stack([k, k]), torch.stack([v, v]))
    assert e.value.status == lf.LF_ERR_STATE
    fill[1].decode_step(q, k, v)  # level again: the group works
    g2.decode_step(torch.stack([q, q]), torch.stack([k, k]), torch.stack([v, v]))
    torch.cuda.synchronize()
    g2.close()
    for c in att + twin + other + fill:
        c.close()


# ------------------------------------------------------------------ explicit validity mask (Alg. 1's M)

def _random_mask(wl, seed, density):
    rng = np.random.default_rng(seed)
    m = rng.random((wl.batch, wl.kv_heads, wl.budget)) < density
    m[..., wl.budget // 3] = True                      # no unit is ever empty
    if wl.units > 1:
        m.reshape(wl.units, -1)[0, :] = True           # one unit without a hole: it evicts from the start
    return m


@pytest.mark.parametrize("name,dtype,B,Hq,Hkv,D,N,flags,density", [
    ("single", "bf16", 48, 16, 4, 128, 300, 0, 0.9),            # one workgroup per unit
    ("coop", "bf16", 2, 28, 4, 128, 2048, 0, 0.98),             # several workgroups per unit
    ("coop-sparse", "bf16", 1, 8, 2, 128, 1100, 0, 0.3),        # whole tiles and workgroup shares invalid
    ("split", "bf16", 3, 8, 2, 128, 700, lf.LF_FLAG_FORCE_SPLIT, 0.9),
    ("split-big", "bf16", 40, 8, 2, 128, 2048, lf.LF_FLAG_FORCE_SPLIT, 0.97),
    ("valu-bf16", "bf16", 2, 6, 2, 128, 333, lf.LF_FLAG_FORCE_VALU, 0.8),
    ("fp32", "f32", 2, 8, 2, 64, 200, 0, 0.7),
])
def test_explicit_mask_holes_fill_first_then_eviction(name, dtype, B, Hq, Hkv, D, N, flags, density):
    # a full cache of which a random subset is valid: the holes take the next tokens lowest
    # first, then the argmin takes over; attention never sees an invalid slot
    wl = _small("mask-" + name, dtype, B, Hq, Hkv, D, N, n_init=N, steps=1, sink_scale=4.0, seed=120)
    mask = _random_mask(wl, 7, density)
    holes = int((~mask).reshape(wl.units, -1).sum(-1).max())
    steps = holes + 12
    units = None if wl.units <= 24 else list(range(0, wl.units, wl.units // 12))
    rep, gpu, ora = run_lockstep(wl, steps=steps, flags=flags, mask=mask, check_scores_every=max(steps // 4, 1),
                                 units=units)
    assert rep.steps == steps and ora.mask().all()
    gpu.close()


def test_ragged_batch_through_a_prefix_mask():
    # sequences of different lengths in one batch: rows past a sequence's length are masked
    wl = _small("mask-ragged", "bf16", 6, 16, 4, 128, 256, n_init=200, steps=1, seed=121)
    lens = np.array([200, 1, 17, 128, 199, 64])
    mask = np.arange(wl.budget)[None, None, :] < lens[:, None, None] + np.zeros((1, wl.kv_heads, 1), dtype=int)
    rep, gpu, ora = run_lockstep(wl, steps=300, mask=mask, check_scores_every=50)
    assert ora.mask().all()                            # even the shortest sequence has filled its cache
    gpu.close()


def test_mask_can_be_set_again_mid_run_and_needs_a_compressing_cache():
    wl = _small("mask-again", "bf16", 2, 8, 2, 128, 160, n_init=100, steps=1, seed=122)
    mask = np.arange(wl.budget)[None, None, :] < np.array([100, 40])[:, None, None] + np.zeros((1, 2, 1), dtype=int)
    rep, gpu, ora = run_lockstep(wl, steps=30, mask=mask)
    # drop every third slot of the second sequence, keep going on both sides
    m2 = ora.mask().reshape(wl.batch, wl.kv_heads, wl.budget).astype(bool)
    m2[1, :, ::3] = False
    gpu.set_mask(torch.as_tensor(m2))
    ora.set_mask(m2.reshape(wl.units, 1, wl.budget))
    for t in range(30, 180):
        q, k, v = (W.to_torch(x, wl, "cuda") for x in W.host_step(wl, t, 0))
        out, idx = gpu.decode_step(q, k, v)
        o_ref, i_ref = ora.step(W.to_f64(q).reshape(wl.units, -1, wl.head_dim), W.to_f64(k).reshape(wl.units, 1, -1),
                                W.to_f64(v).reshape(wl.units, 1, -1))
        assert np.abs(W.to_f64(out).reshape(o_ref.shape) - o_ref).max() <= 2e-2
        if compare_indices(idx.cpu().numpy(), i_ref, ora.scores(), ora.mask().reshape(wl.units, -1).all(-1), rep,
                           where=f"re-mask step {t}"):
            ora.set_pending(idx.cpu().numpy().reshape(wl.units, 1))
    assert ora.mask().all()
    gpu.close()
    att = lf.LongFlowCache(2, 8, 2, 128, 64, flags=lf.LF_FLAG_ATTENTION_ONLY,
                           k_init=torch.zeros(2, 2, 64, 128, device="cuda", dtype=torch.bfloat16),
                           v_init=torch.zeros(2, 2, 64, 128, device="cuda", dtype=torch.bfloat16))
    with pytest.raises(lf.LongFlowError) as e:
        att.set_mask(torch.ones(2, 2, 64))
    assert e.value.status == lf.LF_ERR_UNSUPPORTED
    att.close()


# ------------------------------------------------------------------ batch eviction of the k lowest scores

@pytest.mark.parametrize("name,dtype,B,Hq,Hkv,D,N,n_init,flags,k", [
    ("single", "bf16", 48, 16, 4, 128, 300, 299, 0, 17),
    ("coop", "bf16", 2, 28, 4, 128, 2048, 2047, 0, 128),
    ("filling", "bf16", 2, 8, 2, 128, 600, 200, 0, 50),             # prefix not yet full: the rest turns into holes too
    ("split", "bf16", 3, 8, 2, 128, 700, 699, lf.LF_FLAG_FORCE_SPLIT, 33),
    ("fp32", "f32", 2, 8, 2, 64, 200, 150, 0, 60),                  # vector-ALU path, side array first used here
])
def test_batch_eviction_of_the_k_lowest_scores(name, dtype, B, Hq, Hkv, D, N, n_init, flags, k):
    wl = _small("evict-" + name, dtype, B, Hq, Hkv, D, N, n_init=n_init, steps=1, sink_scale=4.0, seed=130)
    units = None if wl.units <= 24 else list(range(0, wl.units, wl.units // 12))
    rep, gpu, ora = run_lockstep(wl, steps=5, flags=flags, units=units)
    sel = np.arange(wl.units) if units is None else np.asarray(units)
    sc = ora.scores().reshape(len(sel), N)                         # scores of the last step, float64
    valid = ora.mask().reshape(len(sel), N).astype(bool)
    pend = ora.pending().reshape(-1)
    ev_gpu = gpu.evict_lowest(k).cpu().numpy().reshape(wl.units, k)[sel]
    ev_ref = ora.evict_lowest(k).reshape(len(sel), k)
    steer = ora.mask().reshape(len(sel), N).astype(bool)
    for u in range(len(sel)):
        g = ev_gpu[u]
        assert len(set(g.tolist())) == k and valid[u, g].all()     # k distinct valid slots
        if valid[u].all():
            assert g[0] == pend[u]                                 # the slot the last step chose goes first
        s_g = sc[u, g]
        assert (np.diff(s_g) >= -1e-6 * np.abs(s_g[1:])).all()      # ascending score, up to near-ties
        if set(g.tolist()) != set(ev_ref[u].tolist()):             # differing sets: only across a near-tie
            kth = np.sort(sc[u, valid[u]])[k - 1]
            odd = np.array(sorted(set(g.tolist()) ^ set(ev_ref[u].tolist())))
            assert (np.abs(sc[u, odd] - kth) <= 1e-6 * kth).all(), f"unit {u}: {odd} are no near-ties of the k-th score"
            rep.near_ties += 1
            steer[u] = valid[u]
            steer[u, g] = False
    ora.set_mask(steer.reshape(len(sel), 1, N))                     # same holes on both sides from here on
    holes = int((~steer).sum(-1).max())
    rep, gpu, ora = run_lockstep(wl, steps=holes + 8, gpu_cache=gpu, oracle_cache=ora, t0=5, units=units, report=rep,
                                 check_scores_every=holes // 2)
    assert ora.mask().all()
    # argument checks
    with pytest.raises(lf.LongFlowError) as e:
        gpu.evict_lowest(N)
    assert e.value.status == lf.LF_ERR_INVALID_ARG
    fresh = lf.LongFlowCache(1, 2, 1, 128, 64)
    with pytest.raises(lf.LongFlowError) as e:
        fresh.evict_lowest(3)
    assert e.value.status == lf.LF_ERR_STATE
    fresh.close()
    gpu.close()


# ------------------------------------------------------------------ save / resume

@pytest.mark.parametrize("with_holes", [False, True], ids=["full", "holes"])
def test_resume_from_saved_state_continues_bit_identically(with_holes):
    # K/V buffers + validity + the last returned index are the whole state of a cache
    wl = _small("resume", "bf16", 3, 16, 4, 128, 400, n_init=399, steps=1, seed=140)
    k0, v0 = W.host_prefill(wl, 0)
    a = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget,
                         k_init=W.to_torch(k0, wl, "cuda"), v_init=W.to_torch(v0, wl, "cuda"))
    idx = None
    for t in range(6):
        q, k, v = (W.to_torch(x, wl, "cuda") for x in W.host_step(wl, t, 0))
        _, idx = a.decode_step(q, k, v)
    if with_holes:
        a.evict_lowest(9)
        for t in range(6, 9):                        # three of the nine holes refilled
            q, k, v = (W.to_torch(x, wl, "cuda") for x in W.host_step(wl, t, 0))
            _, idx = a.decode_step(q, k, v)
    t0 = 9 if with_holes else 6
    torch.cuda.synchronize()
    b = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget,
                         k_init=a.k_cache.clone(), v_init=a.v_cache.clone())
    b.set_pending(idx.clone())
    if with_holes:
        b.set_mask(a.mask())
        assert int((a.mask() == 0).sum()) == 6 * wl.units
    for t in range(t0, t0 + 20):
        q, k, v = (W.to_torch(x, wl, "cuda") for x in W.host_step(wl, t, 0))
        oa, ia = a.decode_step(q, k, v)
        ob, ib = b.decode_step(q, k, v)
        assert torch.equal(oa.view(torch.int16), ob.view(torch.int16)) and torch.equal(ia, ib), f"step {t}"
    assert torch.equal(a.mask(), b.mask()) and bool(a.mask().all())
    a.close(); b.close()


# ------------------------------------------------------------------ random operation sequences

def _op_sequences(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(count):
        path = int(rng.choice([0, 0, lf.LF_FLAG_FORCE_SPLIT, lf.LF_FLAG_FORCE_UNIT, lf.LF_FLAG_FORCE_VALU]))
        dtype = "f32" if (path == 0 and rng.random() < 0.25) else "bf16"
        D = 64 if dtype == "f32" else 128
        gmax = 8 if path == lf.LF_FLAG_FORCE_VALU else 16
        G = int(rng.integers(1, gmax + 1))
        Hkv = int(rng.integers(1, 3))
        B = int(rng.integers(1, 4))
        N = int(rng.choice([int(rng.integers(40, 300)), int(rng.integers(600, 1500)), int(rng.integers(2000, 2600))]))
        n_init = int(rng.integers(N // 2, N))
        cases.append((dtype, B, G * Hkv, Hkv, D, N, n_init, path if dtype == "bf16" else 0, int(rng.integers(1 << 30))))
    return cases


@pytest.mark.parametrize("case", _op_sequences(10, 20260312), ids=lambda c: "-".join(str(x) for x in c[:8]))
def test_random_operation_sequences(case):
    # decode steps interleaved with batch evictions, re-masking and grouped steps, every
    # result checked against the oracle taken through the same operations
    dtype, B, Hq, Hkv, D, N, n_init, flags, seed = case
    wl = W.Workload("ops", dtype, B, Hq, Hkv, D, N, n_init, 1, sink_scale=4.0 if seed & 1 else 1.0, seed=seed)
    rng = np.random.default_rng(seed)
    rep, gpu, ora = run_lockstep(wl, steps=3, flags=flags)
    # a second cache of the same geometry rides along in the grouped steps (its content is not checked)
    k0, v0 = W.host_prefill(wl, 1)
    other = lf.LongFlowCache(B, Hq, Hkv, D, N, dtype=W.torch_dtype(wl), flags=flags,
                             k_init=W.to_torch(k0, wl, "cuda"), v_init=W.to_torch(v0, wl, "cuda"))
    for t in range(3):
        other.decode_step(*(W.to_torch(x, wl, "cuda") for x in W.host_step(wl, t, 1)))
    group = None
    t = 3
    units = wl.units
    done = {"steps": 0, "evict": 0, "mask": 0, "group": 0}
    for _ in range(14):
        op = str(rng.choice(["steps", "steps", "evict", "mask", "group"]))
        if op == "evict":
            k = int(rng.integers(1, max(2, min(24, N // 8))))
            sc = ora.scores().reshape(units, N)
            valid = ora.mask().reshape(units, N).astype(bool)
            ev = gpu.evict_lowest(k).cpu().numpy().reshape(units, k)
            ev_ref = ora.evict_lowest(k).reshape(units, k)
            steer = ora.mask().reshape(units, N).astype(bool)
            for u in range(units):
                got, want = set(ev[u][ev[u] >= 0].tolist()), set(ev_ref[u][ev_ref[u] >= 0].tolist())
                assert len(got) == len(want)
                if got != want:                       # only across a near-tie of the last score taken
                    kth = np.sort(sc[u, valid[u]])[min(k, valid[u].sum()) - 1]
                    odd = np.array(sorted(got ^ want))
                    assert (np.abs(sc[u, odd] - kth) <= 1e-6 * kth).all()
                    steer[u] = valid[u]
                    steer[u, sorted(got)] = False
            ora.set_mask(steer.reshape(units, 1, N))
            if group is not None:                     # the rider must follow into mask mode
                other.set_mask(torch.ones(B, Hkv, N))
        elif op == "mask":
            m = ora.mask().reshape(units, N).astype(bool)
            drop = rng.random((units, N)) < rng.choice([0.01, 0.1])
            drop[:, int(rng.integers(N))] = False
            keep = m & ~drop
            keep[np.arange(units), np.argmax(m, axis=1)] = True   # never empty
            gpu.set_mask(torch.as_tensor(keep.reshape(B, Hkv, N)))
            ora.set_mask(keep.reshape(units, 1, N))
            other.set_mask(torch.ones(B, Hkv, N))
        elif op == "group":
            if group is None:
                if gpu.valid_count != other.valid_count:
                    continue
                try:
                    group = lf.LongFlowGroup([gpu, other])
                except lf.LongFlowError:                # one masked, the other not
                    other.set_mask(torch.ones(B, Hkv, N))
                    if gpu.valid_count != other.valid_count:
                        continue
                    group = lf.LongFlowGroup([gpu, other])
            n_steps = int(rng.integers(1, 4))
            member = _GroupMember(group, 0, wl, seed=seed + t)
            try:
                rep, _, ora = run_lockstep(wl, steps=n_steps, gpu_cache=member, oracle_cache=ora, t0=t, report=rep,
                                           check_scores_every=2)
            except lf.LongFlowError as e:               # the members drifted apart in fill level or mode
                assert e.status == lf.LF_ERR_STATE
                continue
            t += n_steps
            done["group"] += n_steps
            continue
        else:
            n_steps = int(rng.integers(1, 6))
            rep, _, ora = run_lockstep(wl, steps=n_steps, gpu_cache=gpu, oracle_cache=ora, t0=t, report=rep,
                                       check_scores_every=3)
            t += n_steps
        done[op] += 1
    print(f"\nops {done} decisions {rep.decisions} near-ties {rep.near_ties}")
    if group is not None:
        group.close()
    gpu.close()
    other.close()


# ------------------------------------------------------------------ max-free softmax (Alg. 1 as printed), attention only

def test_max_free_softmax_equals_the_referenced_one_until_it_overflows():
    wl = _small("maxfree", "bf16", 4, 28, 4, 128, 3000, n_init=3000, steps=1, sink_scale=4.0, seed=17)
    k0, v0 = W.device_prefill(wl, "cuda")
    q, _, _ = W.device_step(wl, 0, "cuda")
    mk = lambda flags, k: lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, 128, wl.budget, flags=flags, k_init=k, v_init=v0)
    AO = lf.LF_FLAG_ATTENTION_ONLY
    ref, mf = mk(AO, k0), mk(AO | lf.LF_FLAG_MAX_FREE, k0)
    o_ref, _ = ref.decode_step(q)
    o_mf, _ = mf.decode_step(q)
    torch.cuda.synchronize()
    # both against the oracle on a few units, and against each other
    G, D = wl.group, 128
    for u in (0, 5, wl.units - 1):
        out, _, _ = oracle.attend_unit(W.to_f64(q.reshape(wl.units, G, D)[u]), W.to_f64(k0.reshape(wl.units, -1, D)[u]),
                                       W.to_f64(v0.reshape(wl.units, -1, D)[u]))
        for o in (o_ref, o_mf):
            assert np.abs(W.to_f64(o.reshape(wl.units, G, D)[u]) - out).max() <= 2e-2
    assert (o_ref.float() - o_mf.float()).abs().max().item() <= 2 ** -7
    # keys scaled until a logit passes the fp32 range of exp: the reference keeps the default finite
    # and right, the printed form has nothing to hold on to
    kbig = (k0.float() * 64).to(torch.bfloat16)
    ref2, mf2 = mk(AO, kbig), mk(AO | lf.LF_FLAG_MAX_FREE, kbig)
    o_ref2, _ = ref2.decode_step(q)
    o_mf2, _ = mf2.decode_step(q)
    torch.cuda.synchronize()
    logits = (q.float().reshape(wl.batch, wl.kv_heads, G, D) @ kbig.float().transpose(-1, -2)) / np.sqrt(D)
    assert logits.max().item() > 100
    assert torch.isfinite(o_ref2.float()).all()
    out, _, _ = oracle.attend_unit(W.to_f64(q.reshape(wl.units, G, D)[0]), W.to_f64(kbig.reshape(wl.units, -1, D)[0]),
                                   W.to_f64(v0.reshape(wl.units, -1, D)[0]))
    assert np.abs(W.to_f64(o_ref2.reshape(wl.units, G, D)[0]) - out).max() <= 2e-2
    assert not torch.isfinite(o_mf2.float()).all()
    # the variant exists on the fused matrix-core kernel only
    with pytest.raises(lf.LongFlowError):
        lf.LongFlowCache(1, 4, 1, 128, 64, flags=lf.LF_FLAG_MAX_FREE | lf.LF_FLAG_FORCE_SPLIT)
    with pytest.raises(lf.LongFlowError):
        lf.LongFlowCache(1, 4, 1, 64, 64, flags=AO | lf.LF_FLAG_MAX_FREE, k_init=k0[:1, :1, :8, :64].contiguous(), v_init=v0[:1, :1, :8, :64].contiguous())


@pytest.mark.parametrize("B,N,n_init,steps", [(48, 1500, 1490, 40), (2, 2100, 0, 2140), (1, 700, 690, 30)],
                         ids=["one_workgroup_per_unit", "several_from_empty", "several_small"])
def test_max_free_softmax_in_the_evicting_step(B, N, n_init, steps):
    # Alg. 1 as printed (no running reference) on the whole step: same outputs, decisions and scores as the
    # oracle.  The sink key (x4) drives some logits past the window in which the 8-bit codes have two-sided
    # bounds, so the one-sided ones are exercised too.
    wl = _small("maxfree_evict", "bf16", B, 28, 4, 128, N, n_init=n_init, steps=steps, sink_scale=4.0, seed=23)
    rep, gpu, _ = run_lockstep(wl, flags=lf.LF_FLAG_MAX_FREE, check_scores_every=7, host_inputs=False)
    print(f"\n{wl.name}: {rep.steps} steps, {rep.decisions} decisions, {rep.near_ties} near-ties, "
          f"max|out-oracle| {rep.max_out_err:.2e}, max score rel {rep.max_score_rel:.2e}")
    # a mask, batch eviction and groups are not offered for the variant
    with pytest.raises(lf.LongFlowError) as e:
        gpu.set_mask(torch.ones((wl.batch, wl.kv_heads, N), dtype=torch.uint8))
    assert e.value.status == lf.LF_ERR_UNSUPPORTED
    with pytest.raises(lf.LongFlowError) as e:
        gpu.evict_lowest(2)
    assert e.value.status == lf.LF_ERR_UNSUPPORTED
    gpu.close()


@pytest.mark.parametrize("dtype,D,flags", [("bf16", 128, 0), ("bf16", 128, lf.LF_FLAG_FORCE_SPLIT), ("f32", 64, 0)],
                         ids=["unit", "split", "valu"])
def test_a_padded_sequence_of_zero_rows_decides_exactly_and_quickly(dtype, D, flags):
    # one sequence of the batch is padding: every K and V row zero, so every score is an exact 0 and the
    # lowest slot goes each step; the other sequences are ordinary.  (All of its slots are eviction
    # candidates -- the decision must not fall back to re-scoring each of them.)
    wl = _small("padded", dtype, 3, 8, 2, D, 4096, n_init=4096, steps=6, sink_scale=4.0, seed=61)
    k0, v0 = W.device_prefill(wl, "cuda")
    k0[1] = 0
    v0[1] = 0
    gpu = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, D, wl.budget, dtype=W.torch_dtype(wl), flags=flags, k_init=k0, v_init=v0)
    ora = oracle.OracleCache(wl.units, wl.group, 1, D, wl.budget)
    ora.init(W.to_f64(k0.reshape(wl.units, 1, wl.budget, D)), W.to_f64(v0.reshape(wl.units, 1, wl.budget, D)))
    first = torch.full((wl.batch, wl.kv_heads), 5, dtype=torch.int32)
    gpu.set_pending(first)
    ora.set_pending(first.numpy().reshape(wl.units, 1))
    import time
    times = []
    for t in range(6):
        q, k, v = W.device_step(wl, t, "cuda")
        k[1] = 0
        v[1] = 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out, idx = gpu.decode_step(q, k, v)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
        o_ref, i_ref = ora.step(W.to_f64(q.reshape(wl.units, wl.group, D)), W.to_f64(k.reshape(wl.units, 1, D)),
                                W.to_f64(v.reshape(wl.units, 1, D)))
        assert np.abs(W.to_f64(out.reshape(wl.units, wl.group, D)) - o_ref).max() <= OUT_TOL[dtype]
        assert (idx.reshape(-1).cpu().numpy() == i_ref.reshape(-1)).all(), f"step {t}"
        assert (idx[1] == 0).all()                      # the padded sequence: lowest slot, every time
    assert min(times[1:]) < 4e-4, times                # re-scoring 4096 slots one by one takes about a millisecond
