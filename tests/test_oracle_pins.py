"""Pins for the CPU oracle: things fixed by the paper's definitions and by mathematics,
none of them produced by the oracle itself (hand-worked fractions, closed forms, dense
numpy / library routines on tiny inputs, invariants).  CPU only."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


# --------------------------------------------------------------------------------------
# independent dense numpy statements of each stage (vectorised; tiny inputs only)
# --------------------------------------------------------------------------------------
def np_attention(K, Q, scale):
    """alpha [Hq][W][L]: causal softmax of the last-W queries over all keys."""
    Hkv, L, d = K.shape
    Hq, W, _ = Q.shape
    G = Hq // Hkv
    Kg = np.repeat(K.astype(np.float64), G, axis=0)
    S = scale * np.einsum("hwd,hld->hwl", Q.astype(np.float64), Kg)
    pos = (L - W + np.arange(W))[None, :, None]
    S = np.where(np.arange(L)[None, None, :] <= pos, S, -np.inf)
    S = S - S.max(axis=-1, keepdims=True)
    E = np.exp(S)
    return E / E.sum(axis=-1, keepdims=True)


def np_score(K, Q, mod, scale):
    Hkv, L, d = K.shape
    Hq, W, _ = Q.shape
    G = Hq // Hkv
    A = np_attention(K, Q, scale)
    I = A.reshape(Hkv, G * W, L).sum(axis=1) / (G * W)
    other = mod[None, :] != mod[L - W:][:, None]  # [W][L]
    cross = (A * other[None]).sum(axis=(1, 2)) / W
    return I, cross


def np_select(I, W, B):
    key = I.copy()
    key[len(I) - W:] = np.inf
    order = np.argsort(-key, kind="stable")
    return np.sort(order[:B]).astype(np.int32)


def np_match(K, I, kept, mod, mode_cross, tau):
    K = K.astype(np.float64)
    L = K.shape[0]
    nrm = np.linalg.norm(K, axis=1)
    Kn = np.divide(K, nrm[:, None], out=np.zeros_like(K), where=nrm[:, None] > 0)
    U = Kn @ Kn[kept].T  # [L][B]
    elig = np.broadcast_to(I[kept][None, :] <= tau, U.shape).copy()
    if not mode_cross:
        elig &= mod[kept][None, :] == mod[:, None]
    U = np.where(elig, U, -np.inf)
    assign = np.argmax(U, axis=1).astype(np.int32)
    assign[~elig.any(axis=1)] = -1
    assign[kept] = np.arange(len(kept))
    return assign


def np_merge(K, V, kept, assign):
    B, d = len(kept), K.shape[1]
    ko = np.zeros((B, d)); vo = np.zeros((B, d)); cnt = np.zeros(B)
    sel = assign >= 0
    np.add.at(ko, assign[sel], K[sel].astype(np.float64))
    np.add.at(vo, assign[sel], V[sel].astype(np.float64))
    np.add.at(cnt, assign[sel], 1.0)
    return ko / cnt[:, None], vo / cnt[:, None], (cnt - 1).astype(np.int32)


def rand_case(seed, Hq=4, Hkv=2, L=37, W=5, d=8, img=(9, 25)):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((Hkv, L, d)).astype(np.float32)
    V = rng.standard_normal((Hkv, L, d)).astype(np.float32)
    Q = rng.standard_normal((Hq, W, d)).astype(np.float32)
    mod = np.zeros(L, dtype=np.int32)
    mod[img[0]:img[1]] = 1
    return K, V, Q, mod


# --------------------------------------------------------------------------------------
# hand-worked example
# --------------------------------------------------------------------------------------
def _fr(x):
    if isinstance(x, str) and x in ("inf", "-inf"):
        return float(x)
    return float(Fraction(x))


def test_hand_worked_example(oracle):
    fx = json.load(open(os.path.join(HERE, "golden", "hand_worked_example.json")))
    K = np.array(fx["K"], dtype=np.float32)[None]
    V = np.array(fx["V"], dtype=np.float32)[None]
    Q = np.log(np.array(fx["Q_log_of"], dtype=np.float64)).astype(np.float32)[None]
    mod = np.array(fx["modality"], dtype=np.int32)
    I, cross = oracle.score(K, Q, mod, scale=fx["scale"])
    np.testing.assert_allclose(I[0], [_fr(x) for x in fx["importance"]], rtol=3e-7)
    assert cross[0] == pytest.approx(_fr(fx["cross_share"]), rel=3e-7)
    rho, mode = oracle.flow(cross, 0.5)
    assert rho == pytest.approx(_fr(fx["cross_share"]), rel=3e-7) and mode == 1
    assert oracle.flow(cross, 0.6)[1] == 0
    kept = oracle.select(I[0], fx["W"], fx["budget"])
    assert kept.tolist() == fx["kept_idx"]
    for case in fx["cases"]:
        assign, nd = oracle.match(K[0], I[0], kept, mod, case["mode_cross"], _fr(case["tau"]))
        assert assign.tolist() == case["assign"], case["name"]
        assert nd == case["n_dropped"], case["name"]
        ko, vo, _ = oracle.merge(K[0], V[0], kept, assign)
        np.testing.assert_allclose(ko, [[_fr(x) for x in r] for r in case["K_out"]], atol=1e-15)
        np.testing.assert_allclose(vo, [[_fr(x) for x in r] for r in case["V_out"]], atol=1e-15)


# --------------------------------------------------------------------------------------
# score / flow
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("shape", [dict(Hq=4, Hkv=2), dict(Hq=3, Hkv=3), dict(Hq=6, Hkv=1)])
def test_score_matches_dense_numpy(oracle, seed, shape):
    K, V, Q, mod = rand_case(seed, **shape)
    I, cross = oracle.score(K, Q, mod, scale=0.37)
    I_np, cross_np = np_score(K, Q, mod, 0.37)
    np.testing.assert_allclose(I, I_np, rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(cross, cross_np, rtol=1e-12)


def test_score_default_scale_is_inverse_sqrt_head_dim(oracle):
    K, V, Q, mod = rand_case(5, d=16)
    I, _ = oracle.score(K, Q, mod)
    I_np, _ = np_score(K, Q, mod, 0.25)
    np.testing.assert_allclose(I, I_np, rtol=1e-12)


def test_importance_invariants(oracle):
    K, V, Q, mod = rand_case(3, L=50, W=7)
    I, cross = oracle.score(K, Q, mod)
    np.testing.assert_allclose(I.sum(axis=1), 1.0, rtol=1e-13)
    assert (I > 0).all()
    assert ((cross >= 0) & (cross <= 1)).all()
    # the very last token is seen by the last proxy row only: I <= 1/W
    assert (I[:, -1] <= 1.0 / 7 + 1e-15).all()


def test_uniform_attention_closed_form(oracle):
    """Q = 0 makes every causal row uniform: I(i) = (1/W) sum_{r: pos(r) >= i} 1/(pos(r)+1)."""
    L, W, d = 23, 6, 4
    rng = np.random.default_rng(0)
    K = rng.standard_normal((2, L, d)).astype(np.float32)
    Q = np.zeros((4, W, d), dtype=np.float32)
    mod = np.zeros(L, dtype=np.int32); mod[4:15] = 1
    I, cross = oracle.score(K, Q, mod)
    pos = L - W + np.arange(W)
    want = np.array([sum(1.0 / (p + 1) for p in pos if p >= i) / W for i in range(L)])
    np.testing.assert_allclose(I[0], want, rtol=1e-13)
    np.testing.assert_allclose(I[1], want, rtol=1e-13)
    # every window row is text: cross share = mean over rows of (#image keys visible)/(pos+1)
    want_cross = np.mean([11.0 / (p + 1) for p in pos])
    np.testing.assert_allclose(cross, want_cross, rtol=1e-13)


def test_full_window_is_harmonic_numbers(oracle):
    """W = L and Q = 0: I(i) = (H_L - H_i)/L with H the harmonic numbers."""
    L, d = 12, 4
    K = np.ones((1, L, d), dtype=np.float32)
    Q = np.zeros((1, L, d), dtype=np.float32)
    I, _ = oracle.score(K, Q, np.zeros(L, dtype=np.int32))
    H = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, L + 1))])
    np.testing.assert_allclose(I[0], (H[L] - H[:L]) / L, rtol=1e-13)


def test_rho_is_the_literal_ratio_when_every_token_is_a_proxy(oracle):
    """With the whole prompt as query set the cross share is (A_v->t + A_t->v)/A evaluated on
    the dense L x L attention matrix, exactly as the rho equation is written."""
    rng = np.random.default_rng(7)
    L, d, H = 19, 8, 3
    K = rng.standard_normal((H, L, d)).astype(np.float32)
    Q = rng.standard_normal((H, L, d)).astype(np.float32)
    mod = np.zeros(L, dtype=np.int32); mod[3:11] = 1
    _, cross = oracle.score(K, Q, mod)
    A = np_attention(K, Q, 1.0 / np.sqrt(d))  # [H][L][L], row = query
    vis, txt = mod == 1, mod == 0
    want = []
    for h in range(H):
        a_vt = A[h][np.ix_(vis, txt)].sum()
        a_tv = A[h][np.ix_(txt, vis)].sum()
        want.append((a_vt + a_tv) / A[h].sum())
    np.testing.assert_allclose(cross, want, rtol=1e-12)
    rho, _ = oracle.flow(cross, 0.25)
    assert rho == pytest.approx(np.mean(want), rel=1e-12)


def test_rho_symmetries(oracle):
    K, V, Q, mod = rand_case(11)
    _, cross = oracle.score(K, Q, mod)
    _, cross_swapped = oracle.score(K, Q, 1 - mod)
    np.testing.assert_allclose(cross, cross_swapped, rtol=1e-14)
    _, cross_single = oracle.score(K, Q, np.zeros_like(mod))
    assert (cross_single == 0).all()
    # threshold rule: strictly greater means cross-modal
    assert oracle.flow(np.array([0.25, 0.25]), 0.25)[1] == 0
    assert oracle.flow(np.array([0.25, 0.26]), 0.25)[1] == 1


def test_gqa_group_is_mean_of_duplicated_mha(oracle):
    K, V, Q, mod = rand_case(13, Hq=6, Hkv=2)
    I_gqa, cross_gqa = oracle.score(K, Q, mod)
    I_mha, cross_mha = oracle.score(np.repeat(K, 3, axis=0), Q, mod)
    np.testing.assert_allclose(I_gqa, I_mha.reshape(2, 3, -1).mean(axis=1), rtol=1e-13)
    np.testing.assert_allclose(cross_gqa, cross_mha, rtol=1e-13)


# --------------------------------------------------------------------------------------
# select
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(4))
def test_select_matches_stable_argsort(oracle, seed):
    rng = np.random.default_rng(seed)
    L, W = 60, 6
    I = rng.random(L)
    I[rng.integers(0, L, 12)] = I[3]  # ties
    for B in (W, W + 1, 20, L - 1, L):
        kept = oracle.select(I, W, B)
        assert kept.tolist() == np_select(I, W, B).tolist()
        assert len(set(kept.tolist())) == B and (np.diff(kept) > 0).all()
        assert set(range(L - W, L)) <= set(kept.tolist())
        ev = np.setdiff1d(np.arange(L), kept)
        body = kept[kept < L - W]
        if len(ev) and len(body):
            assert I[body].min() >= I[ev].max()


def test_select_tie_prefers_lower_index(oracle):
    I = np.array([0.1, 0.3, 0.3, 0.3, 0.0, 0.0])
    assert oracle.select(I, 2, 4).tolist() == [1, 2, 4, 5]


# --------------------------------------------------------------------------------------
# match
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(3))
@pytest.mark.parametrize("mode_cross", [0, 1])
def test_match_matches_dense_cosine_argmax(oracle, seed, mode_cross):
    K, V, Q, mod = rand_case(seed, L=45, W=4)
    I, _ = oracle.score(K, Q, mod)
    for g in range(K.shape[0]):
        kept = oracle.select(I[g], 4, 14)
        tau = float(np.sort(I[g][kept])[-4])  # a few pivots are sensitive
        assign, nd = oracle.match(K[g], I[g], kept, mod, mode_cross, tau)
        want = np_match(K[g], I[g], kept, mod, mode_cross, tau)
        assert assign.tolist() == want.tolist()
        assert nd == int((want == -1).sum())
        ev = np.setdiff1d(np.arange(45), kept)
        if not mode_cross:
            ok = assign[ev] >= 0
            assert (mod[kept[assign[ev][ok]]] == mod[ev][ok]).all()
        assert (I[g][kept[assign[ev][assign[ev] >= 0]]] <= tau).all()


def test_match_planted_duplicates_and_scale_invariance(oracle):
    K, V, Q, mod = rand_case(21, L=40, W=4)
    I, _ = oracle.score(K, Q, mod)
    kept = oracle.select(I[0], 4, 10)
    ev = np.setdiff1d(np.arange(40), kept)
    Kp = K[0].copy()
    Kp[ev[0]] = 3.0 * Kp[kept[2]]  # positive multiple of a pivot: cosine exactly 1
    Kp[ev[1]] = 0.25 * Kp[kept[7]]
    assign, _ = oracle.match(Kp, I[0], kept, mod, 1, np.inf)
    assert assign[ev[0]] == 2 and assign[ev[1]] == 7
    # multiplying rows by positive powers of two (exact in floating point) changes no assignment
    gains = 2.0 ** np.random.default_rng(0).integers(-2, 3, size=40)
    assign2, _ = oracle.match(Kp * gains[:, None].astype(np.float32), I[0], kept, mod, 1, np.inf)
    assert assign2.tolist() == assign.tolist()


def test_match_gate_and_modes(oracle):
    K, V, Q, mod = rand_case(22, L=40, W=4)
    I, _ = oracle.score(K, Q, mod)
    kept = oracle.select(I[1], 4, 12)
    ev = np.setdiff1d(np.arange(40), kept)
    a_inf, nd_inf = oracle.match(K[1], I[1], kept, mod, 1, np.inf)
    a_big, _ = oracle.match(K[1], I[1], kept, mod, 1, 2.0)
    assert a_inf.tolist() == a_big.tolist() and nd_inf == 0
    a_neg, nd_neg = oracle.match(K[1], I[1], kept, mod, 1, -1.0)
    assert (a_neg[ev] == -1).all() and nd_neg == len(ev)
    assert a_neg[kept].tolist() == list(range(12))
    # one modality only: intra-modal and cross-modal coincide
    one = np.zeros_like(mod)
    assert oracle.match(K[1], I[1], kept, one, 0, np.inf)[0].tolist() == \
        oracle.match(K[1], I[1], kept, one, 1, np.inf)[0].tolist()


def test_match_zero_norm_rows(oracle):
    rng = np.random.default_rng(3)
    K = rng.standard_normal((12, 4)).astype(np.float32)
    K[5] = 0.0   # evicted zero key: all cosines 0 -> first eligible slot
    K[2] = 0.0   # zero pivot: cosine 0 with everybody
    I = np.full(12, 1.0 / 12)
    kept = np.array([2, 8, 10, 11], dtype=np.int32)
    mod = np.zeros(12, dtype=np.int32)
    assign, nd, ub, us = oracle.match(K, I, kept, mod, 1, np.inf, with_margins=True)
    assert assign[5] == 0 and ub[5] == 0.0
    want = np_match(K, I, kept, mod, 1, np.inf)
    assert assign.tolist() == want.tolist()


def np_match_top2(K, I, kept, mod, mode_cross, tau):
    """Best and runner-up cosine of every token over its eligible pivots, from the dense masked matrix
    (the cosine equation and the thresholded argmax of Sensitivity-Adaptive Token Matching): the two
    largest entries of each row, counted with multiplicity; -inf where there is no such entry."""
    K = K.astype(np.float64)
    nrm = np.linalg.norm(K, axis=1)
    Kn = np.divide(K, nrm[:, None], out=np.zeros_like(K), where=nrm[:, None] > 0)
    U = Kn @ Kn[kept].T
    elig = np.broadcast_to(I[kept][None, :] <= tau, U.shape).copy()
    if not mode_cross:
        elig &= mod[kept][None, :] == mod[:, None]
    U = np.where(elig, U, -np.inf)
    top = -np.sort(-U, axis=1)  # descending
    second = top[:, 1] if U.shape[1] > 1 else np.full(len(U), -np.inf)
    return top[:, 0], second


@pytest.mark.parametrize("seed", range(3))
@pytest.mark.parametrize("mode_cross", [0, 1])
def test_match_margins_are_the_top_two_of_the_dense_cosine_matrix(oracle, seed, mode_cross):
    """u_best / u_second decide which GPU mismatches the parity tests excuse: pin both to the dense
    matrix, with a gate that removes some pivots and a modality restriction that removes others."""
    K, V, Q, mod = rand_case(40 + seed, L=45, W=4)
    I, _ = oracle.score(K, Q, mod)
    for g in range(K.shape[0]):
        kept = oracle.select(I[g], 4, 14)
        tau = float(np.sort(I[g][kept])[-4])
        _, _, ub, us = oracle.match(K[g], I[g], kept, mod, mode_cross, tau, with_margins=True)
        wb, ws = np_match_top2(K[g], I[g], kept, mod, mode_cross, tau)
        ev = np.setdiff1d(np.arange(45), kept)
        assert np.allclose(ub[ev], wb[ev], rtol=0, atol=1e-12) and (np.isinf(ub[ev]) == np.isinf(wb[ev])).all()
        assert np.allclose(us[ev], ws[ev], rtol=0, atol=1e-12) and (np.isinf(us[ev]) == np.isinf(ws[ev])).all()
        assert (us[ev] <= ub[ev]).all()
        # pivots are not matched: both margins are -inf for them
        assert np.isneginf(ub[kept]).all() and np.isneginf(us[kept]).all()


def test_match_margins_special_cases(oracle):
    """Exact ties give margin 0 (the runner-up equals the best), a single eligible pivot has no
    runner-up (-inf), no eligible pivot leaves both at -inf, and an earlier, larger candidate that is
    later beaten becomes the runner-up (not the third best)."""
    e = np.eye(4, dtype=np.float32)
    K = np.zeros((9, 4), dtype=np.float32)
    K[0] = e[0]                      # pivot slot 0
    K[1] = 2.0 * e[0]                # pivot slot 1: same direction as slot 0 -> exact tie for every token
    K[2] = e[1]                      # pivot slot 2
    K[3] = e[2]                      # pivot slot 3 (made sensitive below)
    K[4] = 3.0 * e[0]                # evicted: cosine 1 with slots 0 and 1 (tie), 0 with slot 2
    K[5] = e[0] + e[1]               # evicted: cos 1/sqrt2 with slots 0, 1, 2 (three-way tie)
    K[6] = e[1] + 0.5 * e[0]         # evicted: slot 2 best (2/sqrt5), slots 0/1 tie for second (1/sqrt5)
    K[7] = e[2]                      # evicted: only the sensitive pivot points its way
    K[8] = 0.0                       # evicted zero row: every cosine is 0
    I = np.array([0.1, 0.1, 0.1, 0.9, 0, 0, 0, 0, 0], dtype=np.float64)
    kept = np.array([0, 1, 2, 3], dtype=np.int32)
    mod = np.array([0, 0, 1, 0, 0, 0, 1, 1, 0], dtype=np.int32)
    a, nd, ub, us = oracle.match(K, I, kept, mod, 1, 0.5, with_margins=True)  # slot 3 is gated out
    r5 = 1.0 / np.sqrt(5.0)
    assert a[4] == 0 and ub[4] == 1.0 and us[4] == 1.0           # tie -> lower slot, margin 0
    assert a[5] == 0 and abs(ub[5] - np.sqrt(0.5)) < 1e-15 and us[5] == ub[5]
    assert a[6] == 2 and abs(ub[6] - 2 * r5) < 1e-15 and abs(us[6] - r5) < 1e-15
    assert a[7] == 0 and ub[7] == 0.0 and us[7] == 0.0           # all remaining cosines are 0
    assert a[8] == 0 and ub[8] == 0.0 and us[8] == 0.0
    wb, ws = np_match_top2(K, I, kept, mod, 1, 0.5)
    assert np.allclose(ub[4:], wb[4:], atol=1e-15) and np.allclose(us[4:], ws[4:], atol=1e-15)
    # intra-modal: token 6 (image) sees only slot 2 -> no runner-up; token 7 (image) likewise;
    # tokens 4, 5, 8 (text) see slots 0 and 1
    a, nd, ub, us = oracle.match(K, I, kept, mod, 0, 0.5, with_margins=True)
    assert a[6] == 2 and abs(ub[6] - 2 * r5) < 1e-15 and np.isneginf(us[6])
    assert a[7] == 2 and ub[7] == 0.0 and np.isneginf(us[7])
    assert a[4] == 0 and us[4] == 1.0
    wb, ws = np_match_top2(K, I, kept, mod, 0, 0.5)
    assert np.allclose(ub[4:], wb[4:], atol=1e-15)
    assert (np.isneginf(us[4:]) == np.isneginf(ws[4:])).all()
    # nothing eligible: both -inf and the token is dropped
    a, nd, ub, us = oracle.match(K, I, kept, mod, 1, -1.0, with_margins=True)
    assert (a[4:] == -1).all() and nd == 5 and np.isneginf(ub[4:]).all() and np.isneginf(us[4:]).all()
    # descending candidates: the runner-up is the second one seen, not the last one beaten
    K2 = np.zeros((4, 2), dtype=np.float32)
    K2[0] = [1, 0]; K2[1] = [1, 1]; K2[2] = [0, 1]; K2[3] = [4, 1]
    kept2 = np.array([0, 1, 2], dtype=np.int32)
    I2 = np.zeros(4)
    a, nd, ub, us = oracle.match(K2, I2, kept2, np.zeros(4, dtype=np.int32), 1, np.inf, with_margins=True)
    n17 = np.sqrt(17.0)
    assert a[3] == 0 and abs(ub[3] - 4 / n17) < 1e-15 and abs(us[3] - 5 / (n17 * np.sqrt(2.0))) < 1e-15


# --------------------------------------------------------------------------------------
# merge
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(3))
def test_merge_matches_scatter_mean_and_conserves_mass(oracle, seed):
    K, V, Q, mod = rand_case(seed + 30, L=48, W=4)
    I, _ = oracle.score(K, Q, mod)
    kept = oracle.select(I[0], 4, 9)
    tau = float(np.sort(I[0][kept])[-3])
    assign, nd = oracle.match(K[0], I[0], kept, mod, 0, tau)
    ko, vo, nm = oracle.merge(K[0], V[0], kept, assign)
    ko_np, vo_np, nm_np = np_merge(K[0], V[0], kept, assign)
    np.testing.assert_allclose(ko, ko_np, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(vo, vo_np, rtol=1e-13, atol=1e-15)
    assert nm.tolist() == nm_np.tolist()
    assert nm.sum() + nd == 48 - 9
    dropped = assign == -1
    lhs = ((1 + nm)[:, None] * ko).sum(axis=0) + K[0][dropped].astype(np.float64).sum(axis=0)
    np.testing.assert_allclose(lhs, K[0].astype(np.float64).sum(axis=0), rtol=1e-12, atol=1e-12)
    lhs = ((1 + nm)[:, None] * vo).sum(axis=0) + V[0][dropped].astype(np.float64).sum(axis=0)
    np.testing.assert_allclose(lhs, V[0].astype(np.float64).sum(axis=0), rtol=1e-12, atol=1e-12)


def test_merge_full_budget_and_pure_eviction_are_bit_exact(oracle):
    K, V, Q, mod = rand_case(40, L=30, W=3)
    I, _ = oracle.score(K, Q, mod)
    kept = oracle.select(I[0], 3, 30)
    assign, nd = oracle.match(K[0], I[0], kept, mod, 1, np.inf)
    ko, vo, nm = oracle.merge(K[0], V[0], kept, assign)
    assert nd == 0 and (nm == 0).all()
    assert (oracle.round_output(ko, "f32") == K[0]).all() and (oracle.round_output(vo, "f32") == V[0]).all()
    kept = oracle.select(I[0], 3, 8)
    assign, nd = oracle.match(K[0], I[0], kept, mod, 1, -1.0)
    ko, vo, nm = oracle.merge(K[0], V[0], kept, assign)
    assert (ko == K[0][kept]).all() and (vo == V[0][kept]).all() and nd == 22


# --------------------------------------------------------------------------------------
# variants of the ablation study: misaligned strategy, similarity-weighted merge
# --------------------------------------------------------------------------------------
def test_inverted_flow_is_the_opposite_strategy(oracle):
    cross = np.array([0.1, 0.5, 0.3, 0.7])  # mean 0.4
    for theta in (0.25, 0.4, 0.55, -1.0, 2.0):  # 0.4: rho == theta is intra-modal, so its inverse is cross
        rho, mode = oracle.flow(cross, theta)
        rho_i, mode_i = oracle.flow(cross, theta, invert=True)
        assert rho == rho_i == pytest.approx(0.4)
        assert mode == (1 if 0.4 > theta else 0) and mode_i == 1 - mode


def np_merge_weighted(K, V, kept, assign):
    """Dense restatement: a [B x L] weight matrix (1 on the pivot, max(cos, 0) on members), rows normalised."""
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    L, B = len(K), len(kept)
    Wm = np.zeros((B, L))
    norms = np.linalg.norm(K64, axis=1)
    for i in range(L):
        s = assign[i]
        if s < 0:
            continue
        j = kept[s]
        if i == j:
            Wm[s, i] = 1.0
        elif norms[i] > 0 and norms[j] > 0:
            Wm[s, i] = max(K64[i] @ K64[j] / (norms[i] * norms[j]), 0.0)
    tot = Wm.sum(axis=1, keepdims=True)
    return (Wm / tot) @ K64, (Wm / tot) @ V64, tot[:, 0]


@pytest.mark.parametrize("seed", range(3))
def test_weighted_merge_matches_dense_weight_matrix(oracle, seed):
    K, V, Q, mod = rand_case(seed + 60, L=48, W=4)
    I, _ = oracle.score(K, Q, mod)
    kept = oracle.select(I[0], 4, 9)
    assign, nd = oracle.match(K[0], I[0], kept, mod, 1, float(np.sort(I[0][kept])[-3]))
    ko, vo, nm, ws = oracle.merge_weighted(K[0], V[0], kept, assign)
    ko_np, vo_np, ws_np = np_merge_weighted(K[0], V[0], kept, assign)
    np.testing.assert_allclose(ko, ko_np, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(vo, vo_np, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(ws, ws_np, rtol=1e-13)
    _, _, nm_u = oracle.merge(K[0], V[0], kept, assign)
    assert nm.tolist() == nm_u.tolist()
    assert (ws >= 1.0).all() and (ws <= 1.0 + nm + 1e-12).all()  # every weight lies in [0, 1]


def test_weighted_merge_special_cases(oracle):
    rng = np.random.default_rng(7)
    d = 16
    pivot = rng.standard_normal(d).astype(np.float32)
    ortho = rng.standard_normal(d)
    ortho -= (ortho @ pivot) / (pivot @ pivot) * pivot
    K = np.stack([pivot, 2 * pivot, 0.5 * pivot, -pivot, np.zeros(d, np.float32),
                  ortho.astype(np.float32), rng.standard_normal(d).astype(np.float32)]).astype(np.float32)
    V = rng.standard_normal(K.shape).astype(np.float32)
    kept = np.array([0, 6], dtype=np.int32)
    # positive multiples of the pivot weigh 1: the plain mean of rows 0, 1, 2
    assign = np.array([0, 0, 0, -1, -1, -1, 1], dtype=np.int32)
    ko, vo, nm, ws = oracle.merge_weighted(K, V, kept, assign)
    ku, vu, _ = oracle.merge(K, V, kept, assign)
    np.testing.assert_allclose(ko, ku, rtol=1e-12)
    np.testing.assert_allclose(vo, vu, rtol=1e-12)
    assert ws[0] == pytest.approx(3.0) and ws[1] == 1.0
    # an opposite, a zero and an orthogonal key weigh 0 (up to the rounding of the orthogonal one): the pivot stays
    assign = np.array([0, -1, -1, 0, 0, 0, 1], dtype=np.int32)
    ko, vo, nm, ws = oracle.merge_weighted(K, V, kept, assign)
    assert nm[0] == 3 and ws[0] == pytest.approx(1.0, abs=1e-6)
    np.testing.assert_allclose(ko[0], K[0], atol=1e-6)
    np.testing.assert_allclose(vo[0], V[0], atol=1e-5)
    assert (ko[1] == K[6]).all() and (vo[1] == V[6]).all()
    # weights of a slot sum to one: its merged key lies between the smallest and largest member entry
    assign = np.array([0, 0, 0, 0, 0, 0, 0], dtype=np.int32)
    kept1 = np.array([0], dtype=np.int32)
    ko, vo, nm, ws = oracle.merge_weighted(K, V, kept1, assign)
    assert (ko[0] <= K.max(axis=0) + 1e-12).all() and (ko[0] >= K.min(axis=0) - 1e-12).all()


# --------------------------------------------------------------------------------------
# decode-time maintenance: cache append and re-merge
# --------------------------------------------------------------------------------------
def test_cache_append_is_concatenation(oracle):
    """K_t = [K_{t-1}, k_t], V_t = [V_{t-1}, v_t] (Preliminary): after t appends the valid rows are
    the appended tokens in order, the rows behind them are untouched, and a full cache refuses."""
    rng = np.random.default_rng(5)
    Hkv, cap, d = 3, 6, 8
    Kc = np.full((Hkv, cap, d), -7.0, dtype=np.float32)
    Vc = np.full((Hkv, cap, d), -9.0, dtype=np.float32)
    toks = [(rng.standard_normal((Hkv, d)).astype(np.float32), rng.standard_normal((Hkv, d)).astype(np.float32))
            for _ in range(cap)]
    n = 0
    for t, (k, v) in enumerate(toks):
        n = oracle.cache_append(Kc, Vc, n, k, v)
        assert n == t + 1
        want_k = np.concatenate([x[0][:, None, :] for x in toks[:n]], axis=1)
        want_v = np.concatenate([x[1][:, None, :] for x in toks[:n]], axis=1)
        assert (Kc[:, :n] == want_k).all() and (Vc[:, :n] == want_v).all()
        assert (Kc[:, n:] == -7.0).all() and (Vc[:, n:] == -9.0).all()
    before = Kc.copy()
    assert oracle.cache_append(Kc, Vc, n, toks[0][0], toks[0][1]) == -1 and (Kc == before).all()


def _cache_case(seed, Hq=4, Hkv=2, cap=40, n=33, W=4, d=8):
    rng = np.random.default_rng(seed)
    Kc = rng.standard_normal((Hkv, cap, d)).astype(np.float32)
    Vc = rng.standard_normal((Hkv, cap, d)).astype(np.float32)
    Q = rng.standard_normal((Hq, W, d)).astype(np.float32)
    return Kc, Vc, Q


@pytest.mark.parametrize("seed", range(3))
def test_cache_remerge_is_the_method_on_the_cache_rows(oracle, seed):
    """The re-merge against the dense numpy restatements of every stage, run on the valid rows as a
    prompt of one modality: dense causal softmax -> stable argsort -> masked cosine argmax -> scatter mean."""
    Kc, Vc, Q = _cache_case(seed)
    Hkv, cap, d = Kc.shape
    n, W, B = 33, 4, 11
    K0, V0 = Kc.copy(), Vc.copy()
    tau = 0.09
    plan, new_len = oracle.cache_remerge(Kc, Vc, n, Q, B, "f32", tau)
    assert new_len == B and plan["rho"] == 0.0
    mod = np.zeros(n, dtype=np.int32)
    I_np, _ = np_score(K0[:, :n], Q, mod, 1.0 / np.sqrt(d))
    np.testing.assert_allclose(plan["I"], I_np, rtol=1e-12, atol=1e-300)
    for g in range(Hkv):
        kept = np_select(plan["I"][g], W, B)
        assert plan["kept_idx"][g].tolist() == kept.tolist()
        a = np_match(K0[g, :n], plan["I"][g], kept, mod, 1, tau)
        assert plan["assign"][g].tolist() == a.tolist()
        assert plan["n_dropped"][g] == int((a == -1).sum())
        ko, vo, _ = np_merge(K0[g, :n], V0[g, :n], kept, a)
        np.testing.assert_allclose(Kc[g, :B], ko.astype(np.float32), rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(Vc[g, :B], vo.astype(np.float32), rtol=1e-6, atol=1e-7)
    # rows behind the new length are left alone
    assert (Kc[:, B:] == K0[:, B:]).all() and (Vc[:, B:] == V0[:, B:]).all()


def test_cache_remerge_special_cases(oracle):
    Kc, Vc, Q = _cache_case(9)
    K0, V0 = Kc.copy(), Vc.copy()
    n, W = 33, 4
    # budget = length: nothing is evicted, the cache is unchanged bit for bit
    plan, new_len = oracle.cache_remerge(Kc, Vc, n, Q, n, "f32", 0.5)
    assert new_len == n and (Kc == K0).all() and (Vc == V0).all()
    assert plan["kept_idx"][0].tolist() == list(range(n))
    # every pivot gated out: pure eviction, the kept rows move up unchanged; the proxies are always kept
    plan, _ = oracle.cache_remerge(Kc, Vc, n, Q, 10, "f32", -1.0)
    for g in range(Kc.shape[0]):
        kept = plan["kept_idx"][g]
        assert (Kc[g, :10] == K0[g, kept]).all() and (Vc[g, :10] == V0[g, kept]).all()
        assert kept[-W:].tolist() == list(range(n - W, n))
        assert plan["n_dropped"][g] == n - 10
    # it equals the whole-prompt pass on the same rows with one modality, whatever theta says
    Kc, Vc = K0.copy(), V0.copy()
    plan, _ = oracle.cache_remerge(Kc, Vc, n, Q, 12, "bf16", 0.08)
    for theta in (-1.0, 0.25, 2.0):
        ref = oracle.layer_pass(K0[:, :n], V0[:, :n], Q, np.zeros(n, dtype=np.int32), 12, "bf16", theta, 0.08)
        assert (ref["assign"] == plan["assign"]).all() and (ref["kept_idx"] == plan["kept_idx"]).all()
        assert (ref["K_out"] == Kc[:, :12]).all() and (ref["V_out"] == Vc[:, :12]).all()
    # mass conservation of the fold (fp32 rounding only): sum over slots of (1 + members) * row + dropped rows
    Kc, Vc = K0.copy(), V0.copy()
    plan, _ = oracle.cache_remerge(Kc, Vc, n, Q, 9, "f32", np.inf)
    for g in range(Kc.shape[0]):
        cnt = np.bincount(plan["assign"][g], minlength=9).astype(np.float64)
        total = (cnt[:, None] * Kc[g, :9].astype(np.float64)).sum(axis=0)
        np.testing.assert_allclose(total, K0[g, :n].astype(np.float64).sum(axis=0), rtol=0, atol=1e-4)


def test_prefill_merge_then_appends_then_remerge_keeps_the_books(oracle):
    """The life of one cache: merged prompt rows, decoded tokens appended behind them up to capacity,
    then a re-merge back to the budget; lengths follow B -> B + R -> B."""
    K, V, Q, mod = rand_case(31, L=50, W=4)
    B, R = 12, 8
    ref = oracle.layer_pass(K, V, Q, mod, B, "f32", 0.25, 0.1)
    Hkv, _, d = K.shape
    Kc = np.zeros((Hkv, B + R, d), dtype=np.float32)
    Vc = np.zeros_like(Kc)
    Kc[:, :B], Vc[:, :B] = ref["K_out"], ref["V_out"]
    rng = np.random.default_rng(1)
    n = B
    for _ in range(R):
        n = oracle.cache_append(Kc, Vc, n, rng.standard_normal((Hkv, d)).astype(np.float32),
                                rng.standard_normal((Hkv, d)).astype(np.float32))
    assert n == B + R and oracle.cache_append(Kc, Vc, n, Kc[:, 0], Vc[:, 0]) == -1
    tail = Kc[:, B + R - 4:B + R].copy()
    plan, n = oracle.cache_remerge(Kc, Vc, n, Q, B, "f32", np.inf)
    assert n == B
    # the four most recent tokens are the proxies: they survive as the last four rows, unmerged-into or not
    for g in range(Hkv):
        assert plan["kept_idx"][g][-4:].tolist() == list(range(B + R - 4, B + R))
        alone = np.bincount(plan["assign"][g], minlength=B)[-4:] == 1
        assert (Kc[g, B - 4:B][alone] == tail[g][alone]).all()


# --------------------------------------------------------------------------------------
# decode attention over the compacted cache
# --------------------------------------------------------------------------------------
def test_decode_attention_matches_dense_softmax_and_closed_forms(oracle):
    rng = np.random.default_rng(77)
    G, B, d = 3, 37, 16
    q = rng.standard_normal((G, d)).astype(np.float32)
    Kc = rng.standard_normal((B, d)).astype(np.float32)
    Vc = rng.standard_normal((B, d)).astype(np.float32)
    out = oracle.decode_attention(q, Kc, Vc)
    logits = q.astype(np.float64) @ Kc.astype(np.float64).T / np.sqrt(d)
    w = np.exp(logits - logits.max(axis=1, keepdims=True))
    w /= w.sum(axis=1, keepdims=True)
    np.testing.assert_allclose(out, w @ Vc.astype(np.float64), rtol=1e-12, atol=1e-14)
    # a zero query attends uniformly: the mean of the value rows
    np.testing.assert_allclose(oracle.decode_attention(np.zeros((1, d), np.float32), Kc, Vc)[0],
                               Vc.astype(np.float64).mean(axis=0), rtol=1e-13)
    # a single cached row is returned as it is, whatever the query
    np.testing.assert_allclose(oracle.decode_attention(q, Kc[:1], Vc[:1]), np.repeat(Vc[:1].astype(np.float64), G, 0))
    # a key far more aligned with the query than the rest takes all the mass
    Kb = Kc.copy()
    Kb[5] = 100.0 * q[0]
    np.testing.assert_allclose(oracle.decode_attention(q[:1], Kb, Vc)[0], Vc[5], atol=1e-9)
    # an explicit scale of 0 is uniform attention again; permuting the cache rows changes nothing
    np.testing.assert_allclose(oracle.decode_attention(q, Kc, Vc, scale=0.0)[1], Vc.astype(np.float64).mean(axis=0), rtol=1e-13)
    perm = rng.permutation(B)
    np.testing.assert_allclose(oracle.decode_attention(q, Kc[perm], Vc[perm]), out, rtol=1e-12, atol=1e-14)


def test_rounding_to_bf16_is_nearest_even(oracle):
    # bf16 has 8 significant bits: 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0)
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -30, -3.0, 0.0,
                  257.0, 2.0 ** -130, 1e-45])
    y = oracle.round_output(x, "bf16")
    want = np.array([1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -3.0, 0.0, 256.0, 2.0 ** -130, 0.0])
    assert y.tolist() == want.astype(np.float32).tolist()
    # agrees with integer bit rounding of float32 on values that are exactly float32
    rng = np.random.default_rng(0)
    f = rng.standard_normal(4000).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32).view(np.float32)
    assert (oracle.round_output(f.astype(np.float64), "bf16") == r).all()
    z = rng.standard_normal(100)
    assert (oracle.round_output(z, "f32") == z.astype(np.float32)).all()


# --------------------------------------------------------------------------------------
# whole pass
# --------------------------------------------------------------------------------------
def test_layer_pass_equals_stagewise_and_invariants(oracle):
    K, V, Q, mod = rand_case(50, Hq=4, Hkv=2, L=64, W=6, d=8, img=(10, 50))
    B, tau, theta = 16, 0.2, 0.25
    out = oracle.layer_pass(K, V, Q, mod, B, "bf16", theta, tau)
    I, cross = oracle.score(K, Q, mod)
    rho, mode = oracle.flow(cross, theta)
    assert out["rho"] == rho and out["mode"] == mode
    for g in range(2):
        kept = oracle.select(I[g], 6, B)
        assign, nd = oracle.match(K[g], I[g], kept, mod, mode, tau)
        ko, vo, _ = oracle.merge(K[g], V[g], kept, assign)
        assert out["kept_idx"][g].tolist() == kept.tolist()
        assert out["assign"][g].tolist() == assign.tolist()
        assert out["n_dropped"][g] == nd
        assert (out["K_out"][g] == oracle.round_output(ko, "bf16")).all()
        assert (out["V_out"][g] == oracle.round_output(vo, "bf16")).all()
        # every evicted token has exactly one assignment, an eligible slot or -1
        ev = np.setdiff1d(np.arange(64), kept)
        assert ((assign[ev] >= -1) & (assign[ev] < B)).all()
        assert len(kept) == B


def test_head_permutation_permutes_outputs(oracle):
    K, V, Q, mod = rand_case(51, Hq=3, Hkv=3, L=40, W=4)
    a = oracle.layer_pass(K, V, Q, mod, 10, "f32", 0.25, np.inf)
    p = [2, 0, 1]
    b = oracle.layer_pass(K[p], V[p], Q[p], mod, 10, "f32", 0.25, np.inf)
    assert (a["K_out"][p] == b["K_out"]).all() and (a["assign"][p] == b["assign"]).all()
    assert a["rho"] == pytest.approx(b["rho"], rel=1e-14)


def test_workload_generator_is_seeded_and_shaped():
    from paper_2511_05534_amd import workloads as wl
    w = wl.config(0)
    k1, v1, q1 = w.layer_tensors(0)
    k2, v2, q2 = w.layer_tensors(0)
    assert (k1 == k2).all() and (q1 == q2).all()
    assert k1.shape == (4, 320, 64) and q1.shape == (4, 16, 64) and w.budgets == [64]
    assert wl.config(1).budgets == [68] and wl.config(2).budgets == [410] and wl.config(3).budgets == [819]
    w3 = wl.config(3)
    assert w3.total_tokens == 16384 and len(w3.spans[0]) == 17
    w4 = wl.config(4)
    assert w4.batch == 8 and all(2048 <= L <= 8192 for L in w4.seqlens)
    kb, _, _ = wl.config(1, n_layers=1).layer_tensors(0)
    assert (wl.round_to_bf16(kb) == kb).all()
    assert (wl.bf16_from_bits(wl.bf16_bits(kb)) == kb).all()
