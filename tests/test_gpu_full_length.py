"""Full-length oracle parity at the benchmark configurations: the whole timed run of each
large workload (every consecutive evicting step, at full size, in the launch configuration
bench.py times), with the float64 oracle following sampled (layer, batch, KV head) units in
lock-step.  The caches are rewritten in place hundreds of times here -- slots recycled, the
per-slot side array updated by the inserting wave, the candidate lists rebuilt every step --
which the short full-size tests do not reach."""
import numpy as np
import pytest
import torch

from paper_2603_11504_amd import longflow as lf
from paper_2603_11504_amd import workloads as W

from parity import run_lockstep

pytestmark = pytest.mark.gpu


def _report(tag, rep):
    print(f"\n{tag}: steps {rep.steps} decisions {rep.decisions} near-ties {rep.near_ties} "
          f"max|out-oracle| {rep.max_out_err:.2e} max score rel {rep.max_score_rel:.2e}")
    for note in rep.notes:
        print("   ", note)


def _plan(wl):
    return lf.longflow_plan_info(lf.make_config(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, wl.dtype, 0))


def test_cfg2_every_unit_through_the_whole_timed_run():
    wl = W.CONFIGS[2]
    info = _plan(wl)
    assert info.path == lf.LF_PATH_UNIT_MFMA and info.workgroups_per_unit == 2     # what bench.py times
    rep, gpu, _ = run_lockstep(wl, steps=1 + wl.steps, host_inputs=False, check_scores_every=50)
    _report("cfg2, all 128 units, 100 evicting steps", rep)
    assert rep.steps == 1 + wl.steps and rep.decisions == wl.units * (1 + wl.steps)
    gpu.close()
    del gpu
    torch.cuda.empty_cache()


def test_cfg3_sampled_units_of_two_layers_through_all_256_evicting_steps():
    wl = W.CONFIGS[3]
    info = _plan(wl)
    assert info.path == lf.LF_PATH_UNIT_MFMA and info.workgroups_per_unit == 1
    rng = np.random.default_rng(wl.seed + 7)
    total = 0
    for layer in (5, 22):
        units = np.sort(rng.choice(wl.units, size=64, replace=False))
        # the first step completes the fill (and makes the first decision), then 256 evicting ones
        rep, gpu, _ = run_lockstep(wl, steps=1 + wl.steps, host_inputs=False, units=units, layer=layer,
                                   check_scores_every=128)
        _report(f"cfg3 layer {layer}, 64 sampled units, 256 evicting steps", rep)
        assert rep.steps == 1 + wl.steps
        total += rep.decisions
        gpu.close()
        del gpu
        torch.cuda.empty_cache()
    assert total == 2 * 64 * (1 + wl.steps)


def test_cfg4_sampled_units_through_the_whole_timed_run():
    wl = W.CONFIGS[4]
    info = _plan(wl)
    assert info.path == lf.LF_PATH_UNIT_MFMA and info.workgroups_per_unit == 1
    rng = np.random.default_rng(wl.seed + 7)
    units = np.sort(rng.choice(wl.units, size=64, replace=False))
    rep, gpu, _ = run_lockstep(wl, steps=1 + wl.steps, host_inputs=False, units=units, check_scores_every=25)
    _report("cfg4, 64 sampled units, 50 evicting steps", rep)
    assert rep.steps == 1 + wl.steps
    gpu.close()
    del gpu
    torch.cuda.empty_cache()
