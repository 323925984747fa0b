"""Pins for the float64 oracle (CPU only): every check compares the oracle with
something that is NOT the oracle -- a library routine, a closed form, an
identity proved in the paper, brute force, or a second procedure (Alg. 1)."""
import itertools
import math

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import deferred_norm, longflow_oracle as oracle


def _rand_unit(rng, n, D, G, kscale=1.0):
    q = rng.standard_normal((G, D))
    K = rng.standard_normal((n, D)) * kscale
    V = rng.standard_normal((n, D))
    return q, K, V


# ---------------------------------------------------------------- attention output (eq. 1)

@pytest.mark.parametrize("n,D,G", [(1, 64, 1), (7, 64, 4), (33, 128, 7), (256, 128, 5)])
def test_out_matches_library_softmax_attention(n, D, G):
    rng = np.random.default_rng(n * 1000 + D + G)
    q, K, V = _rand_unit(rng, n, D, G, kscale=2.0)
    out, _, alpha = oracle.attend_unit(q, K, V, want_alpha=True)
    w = scipy_softmax(q @ K.T / math.sqrt(D), axis=1)      # textbook eq. 1
    np.testing.assert_allclose(alpha, w, rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(out, w @ V, rtol=1e-11, atol=1e-13)


def test_closed_form_two_tokens():
    # D = 4, q = (2,0,0,0): s_i = k_i[0].  exp(s) = (1, 3)  ->  alpha = (1/4, 3/4).
    q = np.array([[2.0, 0, 0, 0]])
    K = np.array([[0.0, 5, -1, 2], [math.log(3.0), 7, 7, 7]])
    V = np.array([[4.0, 0, 0, 0], [-8.0, 0, 2, -2]])
    out, score, alpha = oracle.attend_unit(q, K, V, want_alpha=True)
    np.testing.assert_allclose(alpha[0], [0.25, 0.75], rtol=1e-15)
    np.testing.assert_allclose(out[0], [1.0 - 6.0, 0.0, 1.5, -1.5], rtol=1e-14, atol=1e-15)
    # eq. 6: alpha * ||v||_1 = 0.25*4, 0.75*12
    np.testing.assert_allclose(score, [1.0, 9.0], rtol=1e-14)


def test_uniform_keys_give_mean_of_values():
    rng = np.random.default_rng(5)
    q, K, V = _rand_unit(rng, 19, 64, 3)
    K[:] = K[0]
    out, score, _ = oracle.attend_unit(q, K, V)
    np.testing.assert_allclose(out, np.broadcast_to(V.mean(0), out.shape), rtol=1e-12, atol=1e-14)
    # all alpha equal -> the score orders tokens by ||v||_1 alone
    assert oracle.argmin(score) == int(np.argmin(np.abs(V).sum(1)))


def test_scale_is_one_over_sqrt_dk():
    # doubling D by zero-padding must change the logits by sqrt(2): checks that the
    # scale is 1/sqrt(d_k) and not 1/d_k or 1
    rng = np.random.default_rng(6)
    q, K, V = _rand_unit(rng, 9, 32, 1)
    qp = np.concatenate([q, np.zeros_like(q)], 1)
    Kp = np.concatenate([K, np.zeros_like(K)], 1)
    Vp = np.concatenate([V, np.zeros_like(V)], 1)
    _, _, a = oracle.attend_unit(q * math.sqrt(2.0), K, V, True)
    _, _, ap = oracle.attend_unit(qp * 2.0, Kp, Vp, True)
    np.testing.assert_allclose(a, ap, rtol=1e-12)


# ---------------------------------------------------------------- score (eq. 6)

def test_alpha_sums_and_score_mass():
    rng = np.random.default_rng(7)
    for G in (1, 4, 7):
        q, K, V = _rand_unit(rng, 50, 128, G)
        _, score, alpha = oracle.attend_unit(q, K, V, True)
        np.testing.assert_allclose(alpha.sum(1), np.ones(G), rtol=1e-13)
        # sum_i score_i / ||v_i||_1 = G   (a mean over heads would give 1, a max < G)
        np.testing.assert_allclose((score / np.abs(V).sum(1)).sum(), G, rtol=1e-12)


def test_score_is_eq6_at_group_one():
    rng = np.random.default_rng(8)
    q, K, V = _rand_unit(rng, 40, 64, 1, kscale=1.5)
    _, score, _ = oracle.attend_unit(q, K, V)
    alpha = scipy_softmax(K @ q[0] / 8.0)
    c = alpha[:, None] * V                               # contribution vectors, eq. 5
    np.testing.assert_allclose(score, np.abs(c).sum(1), rtol=1e-12)   # L1, not L2
    assert not np.allclose(score, np.sqrt((c ** 2).sum(1)))


def test_group_score_is_sum_of_head_scores():
    rng = np.random.default_rng(9)
    q, K, V = _rand_unit(rng, 31, 64, 5)
    _, score, _ = oracle.attend_unit(q, K, V)
    per_head = sum(oracle.attend_unit(q[h:h + 1], K, V)[1] for h in range(5))
    np.testing.assert_allclose(score, per_head, rtol=1e-13)


def test_equal_value_norms_argmin_is_lowest_logit():
    rng = np.random.default_rng(10)
    q, K, V = _rand_unit(rng, 64, 64, 1)
    V = np.sign(V)                                       # every ||v||_1 = D exactly
    _, score, _ = oracle.attend_unit(q, K, V)
    assert oracle.argmin(score) == int(np.argmin(K @ q[0]))


# ---------------------------------------------------------------- App. A.1: leave-one-out identity

@pytest.mark.parametrize("n", [2, 5, 16])
def test_leave_one_out_identity_and_bound(n):
    rng = np.random.default_rng(100 + n)
    D = 16
    q, K, V = _rand_unit(rng, n, D, 1)
    o, score, alpha = oracle.attend_unit(q, K, V, True)
    o, alpha = o[0], alpha[0]
    Vmax = np.linalg.norm(V, axis=1).max()
    for i in range(n):
        keep = [j for j in range(n) if j != i]
        o_wo = oracle.attend_unit(q, K[keep], V[keep])[0][0]   # recomputed from scratch
        c_i = alpha[i] * V[i]
        R = (o - o_wo) - c_i
        np.testing.assert_allclose(R, -alpha[i] / (1 - alpha[i]) * (o - c_i), rtol=1e-9, atol=1e-13)
        assert np.linalg.norm(R) <= 2 * Vmax * alpha[i] / (1 - alpha[i]) * (1 + 1e-12)
        # the score is the L1 norm of that same contribution vector
        np.testing.assert_allclose(score[i], np.abs(c_i).sum(), rtol=1e-12)
        # renormalisation identity alpha^{j,(\i)} = alpha^j / (1 - alpha^i)
        a_wo = oracle.attend_unit(q, K[keep], V[keep], True)[2][0]
        np.testing.assert_allclose(a_wo, alpha[keep] / (1 - alpha[i]), rtol=1e-10)


# ---------------------------------------------------------------- Alg. 1's route: pieces, max-free, masked, normalised last

@pytest.mark.parametrize("B_k", [1, 3, 16, 37])
def test_deferred_normalisation_over_any_partition_equals_definition(B_k):
    rng = np.random.default_rng(200 + B_k)
    n, D = 37, 64
    q, K, V = _rand_unit(rng, n, D, 1)
    o, score, _ = oracle.attend_unit(q, K, V)
    o2, s2, i2 = deferred_norm.attend_in_pieces(q[0], K, V, np.ones(n), B_k)
    np.testing.assert_allclose(o2, o[0], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(s2, score, rtol=1e-12)
    assert i2 == oracle.argmin(score)


def test_deferred_normalisation_with_mask_equals_definition_on_live_rows():
    rng = np.random.default_rng(300)
    n, D, G = 48, 64, 4
    q, K, V = _rand_unit(rng, n, D, G)
    M = rng.random(n) < 0.6
    M[0] = True
    K2, V2 = K.copy(), V.copy()
    K2[~M] = np.nan
    V2[~M] = np.nan                                       # dead rows must not leak
    o, score, _ = oracle.attend_unit(q, K[M], V[M])
    o2, s2 = deferred_norm.attend_in_pieces_group(q, K2, V2, M, 5)
    np.testing.assert_allclose(o2, o, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(s2[M], score, rtol=1e-12)
    assert np.all(s2[~M] == 0.0)


# ---------------------------------------------------------------- argmin

def test_argmin_brute_force_and_ties():
    rng = np.random.default_rng(400)
    for n in (1, 2, 3, 8):
        for _ in range(20):
            x = rng.integers(0, 4, size=n).astype(float)      # many exact ties
            want = min(range(n), key=lambda i: (x[i], i))
            assert oracle.argmin(x) == want
            assert oracle.argmin(x) == int(np.argsort(x, kind="stable")[0])


def test_permuting_slots_permutes_scores_only():
    rng = np.random.default_rng(500)
    n = 6
    q, K, V = _rand_unit(rng, n, 16, 2)
    o, score, _ = oracle.attend_unit(q, K, V)
    for perm in itertools.islice(itertools.permutations(range(n)), 0, 720, 37):
        perm = list(perm)
        o2, s2, _ = oracle.attend_unit(q, K[perm], V[perm])
        np.testing.assert_allclose(o2, o, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(s2, score[perm], rtol=1e-12)
        assert perm[oracle.argmin(s2)] == oracle.argmin(score)


# ---------------------------------------------------------------- static cache behaviour (Sec. 3.4, Fig. 2 left)

def _run_cache(B, Hq, Hkv, D, N, steps, seed, n_init=0):
    rng = np.random.default_rng(seed)
    c = oracle.OracleCache(B, Hq, Hkv, D, N)
    if n_init:
        c.init(rng.standard_normal((B, Hkv, n_init, D)), rng.standard_normal((B, Hkv, n_init, D)))
    else:
        c.init()
    return c, rng


def test_fill_phase_never_evicts():
    B, Hq, Hkv, D, N = 2, 4, 2, 16, 8
    c, rng = _run_cache(B, Hq, Hkv, D, N, 8, 600)
    toks_k = []
    for t in range(N):
        q = rng.standard_normal((B, Hq, D)); k = rng.standard_normal((B, Hkv, D)); v = rng.standard_normal((B, Hkv, D))
        toks_k.append(k)
        out, idx = c.step(q, k, v)
        assert c.count == t + 1
        K, _ = c.kv()
        for s in range(t + 1):                            # token s sits in slot s, untouched
            np.testing.assert_array_equal(K[:, :, s, :], toks_k[s])
        assert np.isnan(K[:, :, t + 1:, :]).all()         # empty slots never written
        assert np.isfinite(out).all()                     # ... and never read
        if t + 1 < N:
            assert (idx == t + 1).all()                   # next slot is the next empty one
        else:
            sc = c.scores()                               # first real decision: at the step that fills
            assert (idx == sc.argmin(-1)).all()


def test_exactly_one_row_changes_and_it_is_the_returned_slot():
    B, Hq, Hkv, D, N = 2, 6, 2, 16, 12
    c, rng = _run_cache(B, Hq, Hkv, D, N, 0, 700, n_init=N - 1)
    q = rng.standard_normal((B, Hq, D)); k = rng.standard_normal((B, Hkv, D)); v = rng.standard_normal((B, Hkv, D))
    _, idx_prev = c.step(q, k, v)                         # completes the fill, first argmin
    for _ in range(30):
        K0, V0 = c.kv()
        q = rng.standard_normal((B, Hq, D)); k = rng.standard_normal((B, Hkv, D)); v = rng.standard_normal((B, Hkv, D))
        _, idx = c.step(q, k, v)
        K1, V1 = c.kv()
        changed = (K0 != K1).any(-1) | (V0 != V1).any(-1)  # [B,Hkv,N]
        assert (changed.sum(-1) == 1).all()
        assert (changed.argmax(-1) == idx_prev).all()     # slot covered now = slot chosen last step
        np.testing.assert_array_equal(np.take_along_axis(K1, idx_prev[..., None, None].astype(np.int64), 2)[:, :, 0], k)
        assert c.count == N
        idx_prev = idx


def test_cache_step_equals_unit_function_on_cache_rows():
    # the stateful driver adds nothing to the mathematics: the newest token is attended
    # to (it is in the cache before attention) and is itself an eviction candidate
    B, Hq, Hkv, D, N = 1, 3, 1, 16, 5
    c, rng = _run_cache(B, Hq, Hkv, D, N, 0, 800)
    for t in range(9):
        q = rng.standard_normal((B, Hq, D)); k = rng.standard_normal((B, Hkv, D)); v = rng.standard_normal((B, Hkv, D))
        out, idx = c.step(q, k, v)
        K, V = c.kv()
        n = c.count
        o2, s2, _ = oracle.attend_unit(q[0], K[0, 0, :n], V[0, 0, :n])
        np.testing.assert_array_equal(out[0], o2)
        assert (K[0, 0, :n] == k[0, 0]).all(-1).any()     # new token is among the attended rows
        if n == N:
            assert idx[0, 0] == oracle.argmin(s2)


def test_full_cache_without_pending_is_an_error_until_set():
    c, rng = _run_cache(1, 2, 1, 8, 4, 0, 900, n_init=4)
    q = rng.standard_normal((1, 2, 8)); k = rng.standard_normal((1, 1, 8)); v = rng.standard_normal((1, 1, 8))
    with pytest.raises(RuntimeError):
        c.step(q, k, v)
    c.set_pending([[2]])
    c.step(q, k, v)
    K, _ = c.kv()
    np.testing.assert_array_equal(K[0, 0, 2], k[0, 0])


# ---------------------------------------------------------------- explicit mask (Alg. 1's M)

def _masked_cache(B, Hq, Hkv, D, N, seed, density):
    """A full-size cache whose valid slots are a random subset; invalid rows stay NaN."""
    rng = np.random.default_rng(seed)
    c = oracle.OracleCache(B, Hq, Hkv, D, N)
    K0 = rng.standard_normal((B, Hkv, N, D)); V0 = rng.standard_normal((B, Hkv, N, D))
    mask = rng.random((B, Hkv, N)) < density
    mask[..., N // 2] = True                              # never an empty unit
    K0[~mask] = np.nan; V0[~mask] = np.nan
    c.init(K0, V0)
    c.set_mask(mask)
    return c, rng, mask


def test_prefix_mask_equals_count_mode():
    B, Hq, Hkv, D, N, n0 = 2, 4, 2, 16, 10, 4
    ca, rng = _run_cache(B, Hq, Hkv, D, N, 0, 1000, n_init=n0)
    Ka, Va = ca.kv()
    cb = oracle.OracleCache(B, Hq, Hkv, D, N)
    cb.init(Ka, Va)                                        # rows >= n0 are NaN: the mask must hide them
    cb.set_mask(np.arange(N)[None, None, :] < n0 + np.zeros((B, Hkv, 1), dtype=int))
    for t in range(25):                                   # through the fill and well into eviction
        q = rng.standard_normal((B, Hq, D)); k = rng.standard_normal((B, Hkv, D)); v = rng.standard_normal((B, Hkv, D))
        oa, ia = ca.step(q, k, v)
        ob, ib = cb.step(q, k, v)
        np.testing.assert_array_equal(oa, ob)
        np.testing.assert_array_equal(ia, ib)
        np.testing.assert_array_equal(ca.scores(), cb.scores())
        np.testing.assert_array_equal(cb.mask()[0, 0], np.arange(N) < min(n0 + t + 1, N))


def test_masked_step_is_library_attention_over_the_valid_rows():
    B, Hq, Hkv, D, N = 2, 6, 2, 16, 24
    c, rng, mask = _masked_cache(B, Hq, Hkv, D, N, 1100, 0.5)
    G = Hq // Hkv
    for t in range(6):
        pend = c.pending()
        q = rng.standard_normal((B, Hq, D)); k = rng.standard_normal((B, Hkv, D)); v = rng.standard_normal((B, Hkv, D))
        out, idx = c.step(q, k, v)
        K, V = c.kv()
        m = c.mask().astype(bool)
        sc = c.scores()
        for b in range(B):
            for g in range(Hkv):
                assert m[b, g, pend[b, g]]                            # the covered slot became valid
                live = np.flatnonzero(m[b, g])
                assert np.isfinite(K[b, g, live]).all() and np.isnan(K[b, g, ~m[b, g]]).all()
                for h in range(G):
                    a = scipy_softmax(K[b, g, live] @ q[b, g * G + h] / math.sqrt(D))
                    np.testing.assert_allclose(out[b, g * G + h], a @ V[b, g, live], rtol=1e-12, atol=1e-14)
                assert (sc[b, g, ~m[b, g]] == 0).all() and (sc[b, g, live] > 0).all()
                # the deferred-normalisation route of Alg. 1 with the same mask agrees on everything
                o2, s2 = deferred_norm.attend_in_pieces_group(q[b, g * G:(g + 1) * G], K[b, g], V[b, g], m[b, g], 7)
                np.testing.assert_allclose(o2, out[b, g * G:(g + 1) * G], rtol=1e-12, atol=1e-14)
                np.testing.assert_allclose(s2, sc[b, g], rtol=1e-12)


def test_holes_are_filled_lowest_first_then_the_minimum_is_evicted():
    B, Hq, Hkv, D, N = 1, 2, 2, 8, 12
    c, rng, mask = _masked_cache(B, Hq, Hkv, D, N, 1200, 0.4)
    holes = [sorted(np.flatnonzero(~mask[0, g]).tolist()) for g in range(Hkv)]
    np.testing.assert_array_equal(c.pending()[0], [h[0] for h in holes])   # set_mask names the first hole
    for t in range(N + 6):
        q = rng.standard_normal((B, Hq, D)); k = rng.standard_normal((B, Hkv, D)); v = rng.standard_normal((B, Hkv, D))
        pend = c.pending()[0].copy()
        _, idx = c.step(q, k, v)
        for g in range(Hkv):
            if holes[g]:
                assert pend[g] == holes[g].pop(0)                      # holes go in ascending order
            want = holes[g][0] if holes[g] else int(np.argmin(c.scores()[0, g]))
            assert idx[0, g] == want
    assert c.mask().all()


def test_scattering_valid_rows_over_slots_changes_nothing_but_their_places():
    rng = np.random.default_rng(1300)
    D, G, n, N = 16, 3, 7, 20
    q, K, V = _rand_unit(rng, n, D, G)
    o, score, _ = oracle.attend_unit(q, K, V)
    for trial in range(5):
        slots = np.sort(rng.choice(N, size=n, replace=False))
        c = oracle.OracleCache(1, G, 1, D, N)
        K0 = np.full((1, 1, N, D), np.nan); V0 = np.full((1, 1, N, D), np.nan)
        # the step inserts one token itself: pre-place the other n-1 at slots[1:]; the
        # inserted one goes to the lowest free slot, wherever that is
        order = rng.permutation(n)
        K0[0, 0, slots[1:]] = K[order[1:]]; V0[0, 0, slots[1:]] = V[order[1:]]
        m = np.zeros((1, 1, N), dtype=bool); m[0, 0, slots[1:]] = True
        last_slot = int(np.flatnonzero(~m[0, 0])[0])
        c.init(K0, V0); c.set_mask(m)
        out, _ = c.step(q[None], K[order[0]][None, None], V[order[0]][None, None])
        np.testing.assert_allclose(out[0], o, rtol=1e-12, atol=1e-14)
        sc = c.scores()[0, 0]
        np.testing.assert_allclose(sc[last_slot], score[order[0]], rtol=1e-12)
        np.testing.assert_allclose(sc[slots[1:]], score[order[1:]], rtol=1e-12)
        assert np.count_nonzero(sc) == n


# ---------------------------------------------------------------- batch eviction of the k lowest scores

def test_evict_lowest_is_a_stable_sort_of_the_last_scores():
    B, Hq, Hkv, D, N = 2, 4, 2, 16, 20
    c, rng = _run_cache(B, Hq, Hkv, D, N, 0, 1400, n_init=N - 1)
    for t in range(5):
        q = rng.standard_normal((B, Hq, D)); k = rng.standard_normal((B, Hkv, D)); v = rng.standard_normal((B, Hkv, D))
        _, idx = c.step(q, k, v)
    sc = c.scores()
    ev = c.evict_lowest(6)
    for b in range(B):
        for g in range(Hkv):
            order = np.lexsort((np.arange(N), sc[b, g]))          # by score, then by index
            np.testing.assert_array_equal(ev[b, g], order[:6])
            assert ev[b, g, 0] == idx[b, g]                      # the slot the step chose goes first
            assert (c.mask()[b, g] == 0).sum() == 6 and not c.mask()[b, g, ev[b, g]].any()
            assert c.pending()[b, g] == ev[b, g].min()            # holes are refilled lowest slot first
    # the next six tokens land in exactly those slots, ascending; then the argmin is back
    for t in range(8):
        pend = c.pending().copy()
        q = rng.standard_normal((B, Hq, D)); k = rng.standard_normal((B, Hkv, D)); v = rng.standard_normal((B, Hkv, D))
        _, idx = c.step(q, k, v)
        if t < 6:
            np.testing.assert_array_equal(pend, np.sort(ev, -1)[..., t])
        else:
            assert c.mask().all()
            np.testing.assert_array_equal(pend, prev_idx)
        prev_idx = idx


def test_evict_lowest_on_a_filling_cache_and_with_ties():
    B, Hq, Hkv, D, N = 1, 2, 1, 8, 12
    c, rng = _run_cache(B, Hq, Hkv, D, N, 0, 1500, n_init=5)
    q = rng.standard_normal((B, Hq, D)); k = rng.standard_normal((B, Hkv, D)); v = np.zeros((B, Hkv, D))
    c.step(q, k, v)                                               # 6 valid rows, the newest with zero value norm
    k2 = rng.standard_normal((B, Hkv, D))
    c.step(q, k2, np.zeros((B, Hkv, D)))                          # 7 valid, two of them score exactly 0
    sc = c.scores()[0, 0]
    assert (sc[5:7] == 0).all() and (sc[:5] > 0).all() and (sc[7:] == 0).all()
    ev = c.evict_lowest(3)[0, 0]
    # only valid slots compete (the empty ones also hold score 0); equal scores go lowest index first
    np.testing.assert_array_equal(ev, [5, 6, int(np.argmin(sc[:5]))])
    np.testing.assert_array_equal(c.mask()[0, 0], np.isin(np.arange(N), [0, 1, 2, 3, 4]) & (np.arange(N) != ev[2]))
    with pytest.raises(ValueError):
        c.evict_lowest(N)


# ---------------------------------------------------------------- comparison rule: accumulated attention
# (the unfused baseline of Fig. 1; Sec. 4.1's description of H2O)

def test_accumulated_rule_against_token_list_bookkeeping_with_library_softmax():
    """A second procedure that knows nothing of slots: a Python list of live tokens, the
    library softmax, per-token running sums; the token with the least sum leaves."""
    rng = np.random.default_rng(77)
    B, Hkv, G, D, N, T = 2, 2, 3, 16, 6, 25
    c = oracle.OracleCache(B, Hkv * G, Hkv, D, N, rule="accumulated_attention")
    c.init()
    live = [[[] for _ in range(Hkv)] for _ in range(B)]      # per unit: list of dicts
    slot_of = [[{} for _ in range(Hkv)] for _ in range(B)]   # token id -> slot
    free = [[list(range(N)) for _ in range(Hkv)] for _ in range(B)]
    for t in range(T):
        q = rng.standard_normal((B, Hkv * G, D)) * 1.5
        k = rng.standard_normal((B, Hkv, D))
        v = rng.standard_normal((B, Hkv, D))
        out, idx = c.step(q, k, v)
        sc = c.scores()
        for b in range(B):
            for g in range(Hkv):
                toks = live[b][g]
                toks.append({"id": t, "k": k[b, g], "v": v[b, g], "acc": 0.0})
                slot_of[b][g][t] = free[b][g].pop(0)
                Km = np.stack([x["k"] for x in toks]); Vm = np.stack([x["v"] for x in toks])
                w = scipy_softmax(q[b, g * G:(g + 1) * G] @ Km.T / math.sqrt(D), axis=1)
                np.testing.assert_allclose(out[b, g * G:(g + 1) * G], w @ Vm, rtol=1e-11, atol=1e-13)
                for j, x in enumerate(toks):
                    x["acc"] += w[:, j].sum()
                    np.testing.assert_allclose(sc[b, g, slot_of[b][g][x["id"]]], x["acc"], rtol=1e-12)
                if len(toks) == N:
                    j = min(range(N), key=lambda j: toks[j]["acc"])
                    gone = toks.pop(j)
                    s = slot_of[b][g].pop(gone["id"])
                    assert idx[b, g] == s, (t, b, g)
                    free[b][g].append(s)
                else:
                    assert idx[b, g] == len(toks)


def test_accumulated_rule_closed_form_with_uniform_attention():
    """All keys zero: every weight is 1/n.  While filling, the token inserted at step j
    holds G (H_t - H_{j-1}) after step t (harmonic numbers); once full the newest token
    has the least and its slot is recycled for ever, the others gaining G/N per step."""
    G, D, N, T = 4, 8, 5, 12
    rng = np.random.default_rng(3)
    c = oracle.OracleCache(1, G, 1, D, N, rule="accumulated_attention")
    c.init()
    H = [0.0]
    for s in range(1, N + 1):
        H.append(H[-1] + 1.0 / s)
    for t in range(1, T + 1):
        out, idx = c.step(rng.standard_normal((1, G, D)), np.zeros((1, 1, D)), rng.standard_normal((1, 1, D)))
        sc = c.scores().ravel()
        if t <= N:
            want = [G * (H[t] - H[j - 1]) for j in range(1, t + 1)] + [0.0] * (N - t)
            assert idx.item() == (t if t < N else N - 1)
        else:
            want = [G * (H[N] - H[j - 1]) + G * (t - N) / N for j in range(1, N)] + [G / N]
            assert idx.item() == N - 1
        np.testing.assert_allclose(sc, want, rtol=1e-13)


def test_accumulated_rule_conserves_attention_mass():
    """Each step hands out exactly G units of weight (every head's weights sum to 1); what
    leaves the books is what the recycled slot held."""
    rng = np.random.default_rng(5)
    B, Hkv, G, D, N = 1, 3, 5, 32, 9
    c = oracle.OracleCache(B, Hkv * G, Hkv, D, N, rule="accumulated_attention")
    k0 = rng.standard_normal((B, Hkv, 4, D)); v0 = rng.standard_normal((B, Hkv, 4, D))
    c.init(k0, v0)
    assert (c.scores() == 0).all()
    prev = c.scores()
    pend = c.pending()
    for t in range(30):
        c.step(rng.standard_normal((B, Hkv * G, D)) * 2, rng.standard_normal((B, Hkv, D)), rng.standard_normal((B, Hkv, D)))
        now = c.scores()
        lost = np.take_along_axis(prev, pend[..., None].astype(np.int64), axis=2)[..., 0]
        np.testing.assert_allclose(now.sum(-1) - prev.sum(-1) + lost, G, rtol=1e-12)
        prev, pend = now, c.pending()


def test_accumulated_rule_leaves_the_longflow_rule_alone_and_takes_no_mask():
    rng = np.random.default_rng(9)
    B, Hkv, G, D, N = 1, 2, 2, 16, 4
    a = oracle.OracleCache(B, Hkv * G, Hkv, D, N)
    b = oracle.OracleCache(B, Hkv * G, Hkv, D, N, rule="accumulated_attention")
    a.init(); b.init()
    differ = False
    for t in range(12):
        q, k, v = rng.standard_normal((B, Hkv * G, D)), rng.standard_normal((B, Hkv, D)), rng.standard_normal((B, Hkv, D))
        oa, ia = a.step(q, k, v)
        ob, ib = b.step(q, k, v)
        if t < N:      # same cache contents while filling: same attention output
            np.testing.assert_array_equal(oa, ob)
        differ |= bool((ia != ib).any())
        # rule 0 is still eq. 6 on the cache rows
        K, V = a.kv()
        n = a.count
        _, sc, _ = oracle.attend_unit(q[0, :G], K[0, 0, :n], V[0, 0, :n])
        np.testing.assert_array_equal(a.scores()[0, 0, :n], sc)
    assert differ                      # the two rules do not pick the same victims
    with pytest.raises(ValueError):
        b.set_mask(np.ones((B, Hkv, N)))
    with pytest.raises(ValueError):
        b.evict_lowest(1)


# ---------------------------------------------------------------- bulk fill = causal multi-query attention

def test_bulk_fill_is_causal_library_attention_and_ends_like_single_steps():
    rng = np.random.default_rng(21)
    B, Hkv, G, D, N, n0 = 2, 2, 3, 16, 12, 3
    k0 = rng.standard_normal((B, Hkv, n0, D)); v0 = rng.standard_normal((B, Hkv, n0, D))
    for T in (1, 4, N - n0):
        c = oracle.OracleCache(B, Hkv * G, Hkv, D, N)
        c.init(k0, v0)
        q = rng.standard_normal((T, B, Hkv * G, D)) * 1.5
        k = rng.standard_normal((T, B, Hkv, D)); v = rng.standard_normal((T, B, Hkv, D))
        out, idx = c.fill(q, k, v)
        assert c.count == n0 + T
        Kall = np.concatenate([k0, k.transpose(1, 2, 0, 3)], axis=2)      # [B,Hkv,n0+T,D]
        Vall = np.concatenate([v0, v.transpose(1, 2, 0, 3)], axis=2)
        for t in range(T):
            n = n0 + t + 1                                               # token t sees itself and everything before
            for b in range(B):
                for g in range(Hkv):
                    w = scipy_softmax(q[t, b, g * G:(g + 1) * G] @ Kall[b, g, :n].T / math.sqrt(D), axis=1)
                    np.testing.assert_allclose(out[t, b, g * G:(g + 1) * G], w @ Vall[b, g, :n], rtol=1e-11, atol=1e-13)
        Kc, Vc = c.kv()
        np.testing.assert_array_equal(Kc[:, :, :n0 + T], Kall)
        np.testing.assert_array_equal(Vc[:, :, :n0 + T], Vall)
        if n0 + T < N:
            assert (idx == n0 + T).all()
        else:  # the cache just became full: the slot is the argmin of the last token's scores
            sc = c.scores()
            assert (idx == sc.argmin(-1)).all()
            _, s_last, _ = oracle.attend_unit(q[-1, 0, :G], Kall[0, 0], Vall[0, 0])
            np.testing.assert_allclose(sc[0, 0], s_last, rtol=1e-13)
    # more tokens than free slots: the surplus evicts, exactly as single steps do
    a = oracle.OracleCache(B, Hkv * G, Hkv, D, N)
    b = oracle.OracleCache(B, Hkv * G, Hkv, D, N)
    a.init(k0, v0); b.init(k0, v0)
    T = N + 5
    q = rng.standard_normal((T, B, Hkv * G, D)); k = rng.standard_normal((T, B, Hkv, D)); v = rng.standard_normal((T, B, Hkv, D))
    out_a, idx_a = a.fill(q, k, v)
    for t in range(T):
        out_b, idx_b = b.step(q[t], k[t], v[t])
        np.testing.assert_array_equal(out_a[t], out_b)
    np.testing.assert_array_equal(idx_a, idx_b)
    np.testing.assert_array_equal(a.kv()[0], b.kv()[0])
    assert a.count == N
    with pytest.raises(ValueError):
        a.fill(q[:0], k[:0], v[:0])


@pytest.mark.parametrize("rule", ["longflow", "accumulated_attention"])
def test_single_slot_budget_returns_the_new_value_row_and_recycles_slot_zero(rule):
    rng = np.random.default_rng(13)
    B, Hkv, G, D = 2, 2, 3, 8
    c = oracle.OracleCache(B, Hkv * G, Hkv, D, 1, rule=rule)
    c.init()
    for t in range(5):
        q = rng.standard_normal((B, Hkv * G, D)); k = rng.standard_normal((B, Hkv, D)); v = rng.standard_normal((B, Hkv, D))
        out, idx = c.step(q, k, v)
        assert (idx == 0).all() and c.count == 1
        np.testing.assert_allclose(out.reshape(B, Hkv, G, D), np.broadcast_to(v[:, :, None], (B, Hkv, G, D)), rtol=1e-15)
        want = G * np.abs(v).sum(-1) if rule == "longflow" else np.full((B, Hkv), float(G))   # one slot holds all the weight
        np.testing.assert_allclose(c.scores()[..., 0], want, rtol=1e-14)


# ---------------------------------------------------------------- a prompt longer than the budget (Sec. 4.1)

def _votes_by_library(qw, K):
    """Observation-window votes with scipy's softmax: qw [W,G,D], K [T,D] -> [T-W]."""
    W, G, D = qw.shape
    T = K.shape[0]
    P = T - W
    vote = np.zeros(P)
    for j in range(W):
        for h in range(G):
            a = scipy_softmax(K[: P + j + 1] @ qw[j, h] / math.sqrt(D))
            vote += a[:P]
    return vote


@pytest.mark.parametrize("pool", [1, 3, 7])
def test_prompt_compression_votes_pooling_and_selection(pool):
    rng = np.random.default_rng(4000 + pool)
    B, Hq, Hkv, D, T, W, keep = 2, 6, 2, 16, 61, 5, 23
    G = Hq // Hkv
    qw = rng.standard_normal((W, B, Hq, D))
    K = rng.standard_normal((B, Hkv, T, D))
    pooled, kept = oracle.compress_prompt(qw, K, keep, pool)
    for b in range(B):
        for g in range(Hkv):
            vote = _votes_by_library(qw[:, b, g * G:(g + 1) * G], K[b, g])
            # every window query hands out one unit of weight per head, part of it inside the window
            assert vote.sum() <= W * G + 1e-9
            ref = np.convolve(vote, np.ones(pool), mode="same") / pool      # zero padding at both ends
            np.testing.assert_allclose(pooled[b, g], ref, rtol=1e-12, atol=1e-15)
            k = kept[b, g]
            assert (np.diff(k) > 0).all()                                   # original order
            assert (k[-W:] == np.arange(T - W, T)).all()                    # the window is always kept
            order = np.lexsort((np.arange(T - W), -ref))                    # largest first, lowest position among equals
            assert set(k[:-W].tolist()) == set(order[: keep - W].tolist())


def test_prompt_compression_closed_forms_and_edges():
    rng = np.random.default_rng(4100)
    B, Hq, Hkv, D, T, W = 1, 2, 1, 8, 40, 4
    qw = rng.standard_normal((W, B, Hq, D))
    # all keys equal: every position a query sees gets the same weight, so prefix votes are all equal
    # (sum over j of 1/(P+j+1) per head) and ties go to the lowest positions
    K = np.tile(rng.standard_normal((1, 1, 1, D)), (1, 1, T, 1))
    pooled, kept = oracle.compress_prompt(qw, K, 10, 1)
    P = T - W
    expect = Hq * sum(1.0 / (P + j + 1) for j in range(W))
    np.testing.assert_allclose(pooled[0, 0], expect, rtol=1e-12)
    assert kept[0, 0].tolist() == list(range(6)) + list(range(P, T))
    # one prefix key aligned with every query and scaled up: it takes (nearly) all the votes and is kept first
    K2 = rng.standard_normal((1, 1, T, D)) * 0.01
    K2[0, 0, 17] = 50.0 * qw[:, 0].sum((0, 1))
    pooled, kept = oracle.compress_prompt(qw, K2, W + 1, 1)
    assert kept[0, 0, 0] == 17 and pooled[0, 0, 17] > 0.9 * W * Hq
    # keep == T keeps everything; keep == W keeps the window only; bad arguments are refused
    _, kept = oracle.compress_prompt(qw, K2, T, 3)
    assert kept[0, 0].tolist() == list(range(T))
    _, kept = oracle.compress_prompt(qw, K2, W, 3)
    assert kept[0, 0].tolist() == list(range(P, T))
    for bad in (dict(keep=W - 1), dict(keep=T + 1), dict(pool=2), dict(pool=0)):
        with pytest.raises(ValueError):
            oracle.compress_prompt(qw, K2, bad.get("keep", 10), bad.get("pool", 1))
