"""Lock-step comparison of the HIP decode path (through the C ABI) with the float64
oracle on the same seeded inputs.  Helper for the GPU tests and the smoke check."""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

from oracle import longflow_oracle as oracle
from paper_2603_11504_amd import longflow as lf
from paper_2603_11504_amd import workloads as W

OUT_TOL = {"f32": 1e-5, "bf16": 2e-2}   # absolute, on the attention output
NEAR_TIE_REL = 1e-6                     # oracle-score gap below which two slots count as tied
# Unfused comparison path: its importance is a running fp32 sum of fp32 attention weights, so
# the decision inherits their error instead of being re-made exactly.  A weight carries the
# logit's rounding (128 fp32 adds of exact bf16 products, times ln 2: a few 1e-6 relative at
# |logit| ~ 30) and the denominator's (~1e-6); a running sum of T <= 10^4 such terms adds up
# to T * 2^-24 ~ 6e-4 in the worst case and ~sqrt(T) * 2^-24 ~ 6e-6 when roundings scatter.
UNFUSED_TIE_REL = 2e-5
UNFUSED_SCORE_RTOL = 2e-5


@dataclass
class ParityReport:
    steps: int = 0
    decisions: int = 0          # (unit, step) eviction decisions compared
    near_ties: int = 0          # mismatches inside the near-tie allowance (oracle steered)
    max_out_err: float = 0.0
    max_score_rel: float = 0.0
    notes: list = field(default_factory=list)


def compare_indices(gpu_idx, ora_idx, ora_scores, full, rep, where="", tie_rel=NEAR_TIE_REL):
    """Bit-exact unless the oracle's own scores of the two slots are within tie_rel (1e-6
    on the LongFlow path) relative.  Returns True if the oracle must be steered to the GPU's choice."""
    gpu_idx = np.asarray(gpu_idx).reshape(-1)
    ora_idx = np.asarray(ora_idx).reshape(-1)
    rep.decisions += gpu_idx.size
    bad = np.nonzero(gpu_idx != ora_idx)[0]
    if bad.size == 0:
        return False
    full = np.broadcast_to(np.asarray(full, dtype=bool).reshape(-1), gpu_idx.shape)   # per unit, or one for all
    assert full[bad].all(), f"{where}: fill-phase slot differs: gpu {gpu_idx[bad]} oracle {ora_idx[bad]}"
    sc = ora_scores.reshape(gpu_idx.size, -1)
    for u in bad:
        sg, so = sc[u, gpu_idx[u]], sc[u, ora_idx[u]]
        assert sg <= so * (1 + tie_rel), (
            f"{where}: unit {u}: gpu evicts slot {gpu_idx[u]} (oracle score {sg:.17g}), "
            f"oracle evicts {ora_idx[u]} (score {so:.17g}); gap {(sg - so) / so:.3e} is no near-tie")
        rep.near_ties += 1
        rep.notes.append(f"{where}: near-tie unit {u}: {gpu_idx[u]} vs {ora_idx[u]} gap {(sg - so) / max(so, 1e-300):.2e}")
    return True


def run_lockstep(wl: W.Workload, steps=None, flags=0, check_scores_every=0, units=None,
                 device="cuda", layer=0, host_inputs=True, gpu_cache=None, report=None, mask=None,
                 oracle_cache=None, t0=0, rule="longflow"):
    """Advance GPU cache and oracle together for `steps` decode steps, comparing each.

    units: optional list of flat (batch*kv_head) unit indices the oracle follows (the GPU
    always runs the whole workload); None = all of them.
    mask: optional bool array [B, Hkv, N], the explicit validity mask both sides are given
    after the prefill (a cache prefilled to N rows first gets slot 0 as pending slot, which
    units without an invalid slot then keep).
    rule: "longflow", or "accumulated_attention" for the unfused comparison path (flags must
    then carry LF_FLAG_UNFUSED_ACCUM).
    oracle_cache, t0: continue an earlier run (its gpu_cache and oracle, both already
    prefilled) with the inputs of steps t0, t0 + 1, ...
    """
    rep = report or ParityReport()
    steps = wl.steps if steps is None else steps
    dt = W.torch_dtype(wl)
    G, D, N = wl.group, wl.head_dim, wl.budget
    all_units = np.arange(wl.units) if units is None else np.asarray(units)
    nu = len(all_units)

    if oracle_cache is not None:
        return _advance(wl, gpu_cache, oracle_cache, rep, t0, steps, all_units, device, layer, host_inputs,
                        check_scores_every, rule)
    # ---- prefill: same bits on both sides
    if host_inputs:
        k0, v0 = W.host_prefill(wl, layer)
        k0_t = None if k0 is None else W.to_torch(k0, wl, device)
        v0_t = None if v0 is None else W.to_torch(v0, wl, device)
    else:
        k0_t, v0_t = W.device_prefill(wl, device, layer)
    gpu = gpu_cache or lf.LongFlowCache(wl.batch, wl.q_heads, wl.kv_heads, D, N, dtype=dt, flags=flags,
                                        device=device, k_init=k0_t, v_init=v0_t)
    ora = oracle.OracleCache(nu, G, 1, D, N, rule=rule)
    if wl.n_init:
        sel = torch.as_tensor(all_units, device=k0_t.device)
        ku = k0_t.reshape(wl.units, wl.n_init, D)[sel].reshape(nu, 1, wl.n_init, D)
        vu = v0_t.reshape(wl.units, wl.n_init, D)[sel].reshape(nu, 1, wl.n_init, D)
        ora.init(W.to_f64(ku), W.to_f64(vu))
    else:
        ora.init()
    del k0_t, v0_t
    if mask is not None:
        mask = np.asarray(mask, dtype=bool).reshape(wl.units, N)
        if wl.n_init == N:
            gpu.set_pending(torch.zeros((wl.batch, wl.kv_heads), dtype=torch.int32))
            ora.set_pending(np.zeros((nu, 1), dtype=np.int32))
        gpu.set_mask(torch.as_tensor(mask.reshape(wl.batch, wl.kv_heads, N)))
        ora.set_mask(mask[all_units].reshape(nu, 1, N))

    return _advance(wl, gpu, ora, rep, t0, steps, all_units, device, layer, host_inputs, check_scores_every, rule)


def _advance(wl, gpu, ora, rep, t0, steps, all_units, device, layer, host_inputs, check_scores_every,
             rule="longflow"):
    G, D, N = wl.group, wl.head_dim, wl.budget
    unfused = rule == "accumulated_attention"
    tie_rel = UNFUSED_TIE_REL if unfused else NEAR_TIE_REL
    score_rtol = UNFUSED_SCORE_RTOL if unfused else 1e-5
    nu = len(all_units)
    tol = OUT_TOL[wl.dtype]
    for t in range(t0, t0 + steps):
        if host_inputs:
            q, k, v = (W.to_torch(x, wl, device) for x in W.host_step(wl, t, layer))
        else:
            q, k, v = W.device_step(wl, t, device, layer)
        out_t, idx_t = gpu.decode_step(q, k, v)
        torch.cuda.synchronize()
        sel = torch.as_tensor(all_units, device=q.device)
        qu = W.to_f64(q.reshape(wl.units, G, D)[sel])
        ku = W.to_f64(k.reshape(wl.units, 1, D)[sel])
        vu = W.to_f64(v.reshape(wl.units, 1, D)[sel])
        o_ref, i_ref = ora.step(qu, ku, vu)
        o_gpu = W.to_f64(out_t.reshape(wl.units, G, D)[sel])
        assert np.isfinite(o_gpu).all(), f"step {t}: non-finite attention output"
        err = float(np.abs(o_gpu - o_ref).max())
        rep.max_out_err = max(rep.max_out_err, err)
        assert err <= tol, f"step {t}: max |out - oracle| = {err:.3e} > {tol}"
        i_gpu = idx_t.reshape(-1)[sel].cpu().numpy()
        # per unit: while it has a free slot the index is that slot, exactly
        full = ora.mask().reshape(nu, N).all(-1)
        if compare_indices(i_gpu, i_ref, ora.scores(), full, rep, where=f"{wl.name} step {t}", tie_rel=tie_rel):
            ora.set_pending(i_gpu.reshape(nu, 1))
        assert gpu.valid_count == ora.count
        if check_scores_every and (t % check_scores_every == 0 or t == t0 + steps - 1):
            s_gpu = gpu.scores().reshape(wl.units, N)[sel].cpu().numpy().astype(np.float64)
            s_ref = ora.scores().reshape(nu, N)
            n = ora.count
            assert (s_gpu[:, n:] == 0).all()
            assert (s_gpu[ora.mask().reshape(nu, N) == 0] == 0).all()     # invalid slots score 0
            m_gpu = gpu.mask().reshape(wl.units, N)[sel].cpu().numpy() if hasattr(gpu, "mask") else None
            assert m_gpu is None or (m_gpu == ora.mask().reshape(nu, N)).all(), f"step {t}: validity differs"
            rel = np.abs(s_gpu[:, :n] - s_ref[:, :n]) / np.maximum(s_ref[:, :n], 1e-30)
            # fp32 result: 1e-5 relative, except where the score itself is below fp32 range
            ok = (rel <= score_rtol) | (s_ref[:, :n] < 1e-35)
            rep.max_score_rel = max(rep.max_score_rel, float(rel[s_ref[:, :n] >= 1e-35].max(initial=0.0)))
            assert ok.all(), f"step {t}: score rel err {rel[~ok].max():.3e}"
        rep.steps += 1
    return rep, gpu, ora
