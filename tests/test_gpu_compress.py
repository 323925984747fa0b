"""GPU parity of the one-shot prompt compression (longflow_compress_prompt) against the oracle:
pooled votes, the kept rows, the cache it leaves behind, and the decode steps that follow."""
import numpy as np
import pytest
import torch

from oracle import longflow_oracle as oracle
from paper_2603_11504_amd import longflow as lf
from paper_2603_11504_amd import workloads as W

from parity import run_lockstep

pytestmark = pytest.mark.gpu

# The votes are fp32 sums of fp32 attention weights.  A weight carries the logit's rounding (128
# fp32 adds of exact bf16 products, times ln 2: a few 1e-6 relative at |logit| ~ 30), the
# rounding of its column's reference + log2 denominator (an fp32 number of magnitude ~ 30:
# 2e-6 absolute in the exponent) and the exponential's own (~1e-6); W * G of them are added.
VOTE_RTOL = 2e-5
TIE_REL = 4e-5   # two rows whose oracle votes are this close may swap places at the threshold


def _wl(name, B, Hq, Hkv, N, **kw):
    return W.Workload(name, "bf16", B, Hq, Hkv, 128, N, 0, 4 * N, **kw)


def _compress_and_compare(wl, T, Wn, keep, pool, units=None, tail_steps=6):
    G, D, N = wl.group, wl.head_dim, wl.budget
    all_units = np.arange(wl.units) if units is None else np.asarray(units)
    nu = len(all_units)
    sel = torch.as_tensor(all_units, device="cuda")
    qw, kp, vp = W.device_prompt(wl, T, Wn, "cuda")
    gpu = lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, D, N, dtype=torch.bfloat16)
    pooled_t, kept_t = gpu.compress_prompt(qw, kp, vp, keep, pool)
    torch.cuda.synchronize()
    assert gpu.valid_count == keep
    P, kpre = T - Wn, keep - Wn

    qw_u = W.to_f64(qw.reshape(Wn, wl.units, G, D)[:, sel])                       # [W, nu, G, D]
    K_u = W.to_f64(kp.reshape(wl.units, T, D)[sel]).reshape(nu, 1, T, D)
    pooled_ref, kept_ref = oracle.compress_prompt(qw_u, K_u, keep, pool)
    pooled_ref, kept_ref = pooled_ref.reshape(nu, P), kept_ref.reshape(nu, keep)
    pooled_gpu = pooled_t.reshape(wl.units, P)[sel].cpu().numpy().astype(np.float64)
    kept_gpu = kept_t.reshape(wl.units, keep)[sel].cpu().numpy()

    max_rel = 0.0
    if P > 0:
        rel = np.abs(pooled_gpu - pooled_ref) / np.maximum(pooled_ref, 1e-30)
        ok = (rel <= VOTE_RTOL) | (pooled_ref < 1e-30)
        max_rel = float(rel[pooled_ref >= 1e-30].max(initial=0.0))
        assert ok.all(), f"pooled votes: rel err {rel[~ok].max():.3e}"
    swaps = 0
    for i in range(nu):
        kg, kr = kept_gpu[i], kept_ref[i]
        assert (np.diff(kg) > 0).all(), "kept rows are not in ascending prompt order"
        assert (kg[kpre:] == np.arange(P, T)).all(), "the observation window is not kept whole"
        if (kg == kr).all():
            continue
        # a different set is accepted only among rows whose oracle votes tie with the threshold
        assert 0 < kpre < P
        thr = np.sort(pooled_ref[i])[P - kpre]                                   # the kpre-th largest
        diff = np.setxor1d(kg[:kpre], kr[:kpre])
        gap = np.abs(pooled_ref[i][diff] - thr) / thr
        assert (gap <= TIE_REL).all(), f"unit {all_units[i]}: kept sets differ at rows {diff} with gaps {gap}"
        swaps += len(diff) // 2

    # the cache: slots [0, keep) hold exactly the kept prompt rows, bit for bit
    idx = kept_t.reshape(wl.units, keep).long()
    for cache, src in ((gpu.k_cache, kp), (gpu.v_cache, vp)):
        want = torch.gather(src.reshape(wl.units, T, D), 1, idx[:, :, None].expand(-1, -1, D))
        got = cache.reshape(wl.units, N, D)[:, :keep]
        assert torch.equal(want.view(torch.int16), got.view(torch.int16))

    # decoding goes on from there as from a cache created with those rows
    rep = None
    if keep < N and tail_steps:
        ora = oracle.OracleCache(nu, G, 1, D, N)
        kk = torch.as_tensor(kept_gpu, device="cuda").long()
        k0 = torch.gather(kp.reshape(wl.units, T, D)[sel], 1, kk[:, :, None].expand(-1, -1, D))
        v0 = torch.gather(vp.reshape(wl.units, T, D)[sel], 1, kk[:, :, None].expand(-1, -1, D))
        ora.init(W.to_f64(k0).reshape(nu, 1, keep, D), W.to_f64(v0).reshape(nu, 1, keep, D))
        rep, _, _ = run_lockstep(wl, steps=tail_steps, units=None if units is None else all_units, gpu_cache=gpu,
                                 oracle_cache=ora, t0=0, host_inputs=False, check_scores_every=2)
    gpu.close()
    print(f"\n{wl.name}: T {T} W {Wn} keep {keep} pool {pool}: {nu} units, max vote rel err {max_rel:.2e}, "
          f"{swaps} rows swapped between near-ties"
          + (f"; then {rep.steps} steps, {rep.decisions} decisions, {rep.near_ties} near-ties, max|out-oracle| {rep.max_out_err:.2e}" if rep else ""))
    return swaps


@pytest.mark.parametrize("pool", [1, 7])
@pytest.mark.parametrize("G", [1, 7, 16])
def test_votes_selection_and_cache_small(G, pool):
    # ragged everywhere: T and the prefix are no multiples of the 16-row tile, the window is no power of two
    wl = _wl(f"cmp_g{G}", 2, 2 * G, 2, 300, channel_scale_range=(0.5, 3.0), seed=9100 + G)
    _compress_and_compare(wl, T=1111, Wn=13, keep=297, pool=pool)


def test_more_columns_than_one_pass_takes():
    # 64 x 7 = 448 query columns: two rounds of 256 per span; several spans
    wl = _wl("cmp_rounds", 1, 14, 2, 2048, sink_scale=4.0, seed=9201)
    _compress_and_compare(wl, T=5000, Wn=64, keep=2047, pool=5)


def test_edges_window_only_everything_and_no_prefix():
    wl = _wl("cmp_edges", 1, 8, 2, 200, seed=9301)
    _compress_and_compare(wl, T=150, Wn=8, keep=8, pool=3)        # only the window survives
    _compress_and_compare(wl, T=150, Wn=8, keep=150, pool=3)      # the prompt fits: every row kept
    _compress_and_compare(wl, T=40, Wn=40, keep=40, pool=1)       # the window is the whole prompt
    _compress_and_compare(wl, T=21, Wn=5, keep=6, pool=1)         # a prefix shorter than two tiles, one row of it kept
    _compress_and_compare(wl, T=300, Wn=1, keep=200, pool=9, tail_steps=0)  # one window row; cache left full


def test_equal_votes_keep_the_lowest_rows():
    # all keys equal: every prefix row gets bit-identical votes, so the first rows win
    B, Hq, Hkv, D, N, T, Wn, keep = 1, 4, 2, 128, 64, 100, 4, 30
    g = torch.Generator(device="cuda").manual_seed(9401)
    row = torch.randn((B, Hkv, 1, D), generator=g, device="cuda").to(torch.bfloat16)
    kp = row.expand(B, Hkv, T, D).contiguous()
    vp = torch.randn((B, Hkv, T, D), generator=g, device="cuda").to(torch.bfloat16)
    qw = torch.randn((Wn, B, Hq, D), generator=g, device="cuda").to(torch.bfloat16)
    gpu = lf.LongFlowCache(B, Hq, Hkv, D, N)
    pooled, kept = gpu.compress_prompt(qw, kp, vp, keep, 1)
    torch.cuda.synchronize()
    P = T - Wn
    want = list(range(keep - Wn)) + list(range(P, T))
    assert kept.cpu().numpy().reshape(B * Hkv, keep).tolist() == [want] * (B * Hkv)
    pooled = pooled.cpu().numpy().reshape(B * Hkv, P)
    assert (pooled == pooled[:, :1]).all()
    expect = (Hq // Hkv) * sum(1.0 / (P + j + 1) for j in range(Wn))   # closed form: uniform weights
    np.testing.assert_allclose(pooled, expect, rtol=1e-5)
    gpu.close()


def test_refusals_leave_the_cache_alone():
    B, Hq, Hkv, D, N, T, Wn = 1, 4, 2, 128, 64, 100, 4
    z = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device="cuda")
    gpu = lf.LongFlowCache(B, Hq, Hkv, D, N)
    for keep, pool, status in ((3, 1, lf.LF_ERR_INVALID_ARG), (65, 1, lf.LF_ERR_INVALID_ARG), (30, 2, lf.LF_ERR_INVALID_ARG),
                               (30, 0, lf.LF_ERR_INVALID_ARG)):
        with pytest.raises(lf.LongFlowError) as e:
            gpu.compress_prompt(z(Wn, B, Hq, D), z(B, Hkv, T, D), z(B, Hkv, T, D), keep, pool)
        assert e.value.status == status and gpu.valid_count == 0
    with pytest.raises(lf.LongFlowError) as e:                      # keep > T
        gpu.compress_prompt(z(Wn, B, Hq, D), z(B, Hkv, 20, D), z(B, Hkv, 20, D), 30, 1)
    assert e.value.status == lf.LF_ERR_INVALID_ARG
    gpu.decode_step(z(B, Hq, D), z(B, Hkv, D), z(B, Hkv, D))
    with pytest.raises(lf.LongFlowError) as e:                      # no longer empty
        gpu.compress_prompt(z(Wn, B, Hq, D), z(B, Hkv, T, D), z(B, Hkv, T, D), 30, 1)
    assert e.value.status == lf.LF_ERR_STATE and gpu.valid_count == 1
    gpu.close()
    f32 = lf.LongFlowCache(B, Hq, Hkv, 64, N, dtype=torch.float32)
    with pytest.raises(lf.LongFlowError) as e:
        f32.compress_prompt(torch.zeros((Wn, B, Hq, 64), device="cuda"), torch.zeros((B, Hkv, T, 64), device="cuda"),
                            torch.zeros((B, Hkv, T, 64), device="cuda"), 30, 1)
    assert e.value.status == lf.LF_ERR_UNSUPPORTED
    f32.close()


def test_long_prompt_into_a_target_sized_cache():
    # the geometry of the 28-layer target workload (64 x 4 units, 7 heads a group, 8192 slots), a prompt four
    # times the budget, SnapKV's usual window and pooling width; the oracle follows a sample of units
    wl = W.scaled(W.CONFIGS[3], n_init=0, layers=1)
    rng = np.random.default_rng(9501)
    units = np.sort(rng.choice(wl.units, size=12, replace=False))
    _compress_and_compare(wl, T=32768, Wn=32, keep=wl.budget - 1, pool=7, units=units, tail_steps=3)
