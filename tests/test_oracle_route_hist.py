"""Pins for the oracle's route / coact_hist: brute force, closed forms, library special cases."""
import math

import numpy as np
import pytest

from oracle import semmoe_oracle as O
import workloads as WL


def _rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ route_logits
def test_logits_entry_by_entry_loops():
    """a transposed operand, a dropped bias or a wrong class row fails this"""
    r = _rng(1)
    T, d, E, C = 5, 7, 6, 3
    X = r.standard_normal((T, d)).astype(np.float32)
    W = r.standard_normal((E, d)).astype(np.float32)
    b = r.standard_normal(E).astype(np.float32)
    cb = r.standard_normal((C, E)).astype(np.float32)
    tc = np.array([0, 2, -1, 1, 2], dtype=np.int32)
    L = O.route_logits(X, W, b, tc, cb)
    for i in range(T):
        for e in range(E):
            acc = math.fsum(float(X[i, c]) * float(W[e, c]) for c in range(d)) + float(b[e])
            if tc[i] >= 0:
                acc += float(cb[tc[i], e])
            assert L[i, e] == np.float32(acc)
    assert L.dtype == np.float32


# ------------------------------------------------------------------ softmax top-k
def test_softmax_topk_matches_full_sort_and_textbook_softmax():
    r = _rng(2)
    L = r.standard_normal((40, 12)).astype(np.float32)
    ids, w = O.select_topk(L, 3, "softmax", renorm=False)
    for i in range(40):
        full = np.argsort(-L[i].astype(np.float64), kind="stable")
        assert list(ids[i]) == list(full[:3])
        p = np.exp(L[i].astype(np.float64))
        p /= p.sum()
        np.testing.assert_allclose(w[i], p[ids[i]], rtol=1e-13)


def test_softmax_ties_go_to_lower_index_and_descending_order():
    L = np.array([[1.0, 3.0, 3.0, 0.5, 3.0, 2.0],
                  [0.0, 0.0, 0.0, 0.0, 0.0, 0.0]], dtype=np.float32)
    ids, w = O.select_topk(L, 4, "softmax", renorm=True)
    assert list(ids[0]) == [1, 2, 4, 5]
    assert list(ids[1]) == [0, 1, 2, 3]
    np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(w[1], 0.25, rtol=1e-14)


def test_softmax_renorm_equals_softmax_over_selected():
    """softmax over all then renormalise == softmax over the k chosen logits"""
    r = _rng(3)
    L = (3 * r.standard_normal((20, 16))).astype(np.float32)
    ids, w = O.select_topk(L, 4, "softmax", renorm=True)
    for i in range(20):
        z = np.exp(L[i, ids[i]].astype(np.float64))
        np.testing.assert_allclose(w[i], z / z.sum(), rtol=1e-12)


def test_k_equals_E_is_a_permutation_and_weights_sum_to_one():
    r = _rng(4)
    L = r.standard_normal((8, 9)).astype(np.float32)
    ids, w = O.select_topk(L, 9, "softmax", renorm=False)
    for i in range(8):
        assert sorted(ids[i]) == list(range(9))
    np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=1e-13)


def test_permuting_experts_permutes_ids():
    r = _rng(5)
    L = r.standard_normal((16, 10)).astype(np.float32)      # continuous values: no ties
    perm = r.permutation(10)
    ids, w = O.select_topk(L, 3, "softmax", renorm=True)
    ids2, w2 = O.select_topk(L[:, perm], 3, "softmax", renorm=True)
    assert (perm[ids2] == ids).all()
    np.testing.assert_allclose(w2, w, rtol=1e-13)


def test_large_logits_do_not_overflow():
    L = np.array([[1000.0, 999.0, -1000.0]], dtype=np.float32)
    ids, w = O.select_topk(L, 2, "softmax", renorm=False)
    assert list(ids[0]) == [0, 1]
    np.testing.assert_allclose(w[0], [1 / (1 + math.exp(-1)), math.exp(-1) / (1 + math.exp(-1))], rtol=1e-12)


# ------------------------------------------------------------------ sigmoid recipe
def test_sigmoid_f32_close_to_exact_sigmoid():
    x = np.linspace(-35, 35, 200001).astype(np.float32)
    s = O.sigmoid_f32(x)
    xc = np.clip(x.astype(np.float64), -30, 30)
    exact = 1.0 / (1.0 + np.exp(-xc))
    rel = np.abs(s.astype(np.float64) - exact) / exact
    # the rounding of t = -x*log2(e) near |t| = 43 alone costs ~1.3e-6 relative on the tiny tail values
    assert rel.max() < 3e-6
    assert np.abs(s.astype(np.float64) - exact).max() < 1.5e-7      # ~2 ulp of 0.5..1
    assert s.dtype == np.float32
    assert (np.diff(s.astype(np.float64)) >= -2e-7).all()


def test_sigmoid_f32_special_values():
    s = O.sigmoid_f32(np.array([0.0, 30.0, -30.0, 100.0, -100.0], dtype=np.float32))
    assert s[0] == np.float32(0.5)
    assert s[1] == s[3] and s[2] == s[4]
    assert abs(float(s[2]) - math.exp(-30)) / math.exp(-30) < 3e-6


def test_sigmoid_f32_is_scalar_step_by_step():
    """the vectorised recipe equals the same steps done one scalar at a time with explicit rounding"""
    r = _rng(6)
    xs = (8 * r.standard_normal(300)).astype(np.float32)
    f32 = np.float32
    coef = [1.0, 0.6931471805599453, 0.2402265069591007, 0.05550410866482158, 0.009618129107628477,
            0.0013333558146428443, 0.00015403530393381608]
    for x in xs:
        xx = min(max(float(x), -30.0), 30.0)
        t = float(f32(-xx) * f32(1.4426950408889634))
        n = float(np.rint(f32(t)))
        f = float(f32(t) - f32(n))
        p = float(f32(coef[6]))
        for i in range(5, -1, -1):
            p = float(f32(f32(p) * f32(f)))          # product rounded to fp32
            p = float(f32(f32(p) + f32(coef[i])))    # sum rounded to fp32
        z = float(f32(math.ldexp(p, int(n))))
        s = f32(1.0) / f32(f32(1.0) + f32(z))
        assert O.sigmoid_f32(np.array([x]))[0] == s


def _brute_group_limited(sp, s, k, n_group, topk_group):
    E = len(sp)
    gs = E // n_group
    gscore = []
    for g in range(n_group):
        seg = sorted((np.float32(v) for v in sp[g * gs:(g + 1) * gs]), reverse=True)
        gscore.append(np.float32(seg[0] + seg[1]))
    gorder = sorted(range(n_group), key=lambda g: (-gscore[g], g))[:topk_group]
    cand = [e for e in range(E) if e // gs in gorder]
    cand.sort(key=lambda e: (-sp[e], e))
    return cand[:k]


def test_sigmoid_group_limited_against_brute_force():
    r = _rng(7)
    L = (1.5 * r.standard_normal((64, 32))).astype(np.float32)
    bias = (0.1 * r.standard_normal(32)).astype(np.float32)
    ids, w = O.select_topk(L, 4, "sigmoid", renorm=True, n_group=4, topk_group=2, routed_scale=2.5, sel_bias=bias)
    s = O.sigmoid_f32(L)
    sp = s + bias[None, :]
    for i in range(64):
        want = _brute_group_limited(sp[i], s[i], 4, 4, 2)
        assert list(ids[i]) == want
        groups = {e // 8 for e in ids[i]}
        assert len(groups) <= 2 and len(set(ids[i])) == 4
        ws = s[i, ids[i]].astype(np.float64)
        np.testing.assert_allclose(w[i], 2.5 * ws / ws.sum(), rtol=1e-13)   # weights use s, not s + bias
    np.testing.assert_allclose(w.sum(axis=1), 2.5, rtol=1e-13)


def test_sigmoid_single_group_reduces_to_plain_topk_of_logits():
    """sigmoid is monotone: with one group and no bias the ids are the top-k of the logits"""
    r = _rng(8)
    L = (2 * r.standard_normal((50, 24))).astype(np.float32)
    ids, _ = O.select_topk(L, 5, "sigmoid", renorm=True)
    s = O.sigmoid_f32(L)
    for i in range(50):
        full = sorted(range(24), key=lambda e: (-s[i, e], e))
        assert list(ids[i]) == full[:5]


def test_group_score_is_top2_sum_not_max():
    # group 0 has the single largest score, group 1 the larger top-2 sum
    L = np.array([[4.0, -4.0, -4.0, -4.0, 2.0, 2.0, -4.0, -4.0]], dtype=np.float32)
    ids, _ = O.select_topk(L, 2, "sigmoid", renorm=True, n_group=2, topk_group=1)
    assert sorted(ids[0]) == [4, 5]


# ------------------------------------------------------------------ coact_hist
def test_coact_equals_incidence_gram_matrix():
    ids = WL.uniform_random_ids(300, 12, 3, seed=3)
    load, co = O.coact_hist(ids, 12)
    M = np.zeros((300, 12), dtype=np.int64)
    for i in range(300):
        M[i, ids[i]] = 1
    assert (co == M.T @ M).all()
    assert (load == M.sum(axis=0)).all()


def test_coact_closed_forms_and_accumulation():
    T, E, k = 257, 16, 4
    ids = WL.uniform_random_ids(T, E, k, seed=4)
    load, co = O.coact_hist(ids, E)
    assert load.sum() == T * k
    assert (np.diag(co) == load).all()
    assert (co == co.T).all()
    assert co.sum() == T * k * k
    assert (co.sum(axis=1) == k * load).all()
    # streaming two halves accumulates to the same result
    l2, c2 = O.coact_hist(ids[:100], E)
    l2, c2 = O.coact_hist(ids[100:], E, l2, c2)
    assert (l2 == load).all() and (c2 == co).all()


def test_coact_hand_example():
    ids = np.array([[0, 2], [2, 1], [0, 2]], dtype=np.int32)
    load, co = O.coact_hist(ids, 3)
    assert list(load) == [2, 1, 3]
    assert co.tolist() == [[2, 0, 2], [0, 1, 1], [2, 1, 3]]
