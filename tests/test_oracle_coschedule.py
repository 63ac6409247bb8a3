"""Pins of the oracle's co-scheduling solver (Alg. 1 whole, App. B: `expert_place` with its request term,
`req_sched`, the alternation, the token labels) against what the paper and the mathematics fix: the special case
that is the already pinned `place`, hand-worked examples, planted clusters that must be recovered, brute force
over all balanced placements and schedules on tiny inputs, and identities that tie its score and its labels to
functions pinned elsewhere (`local_pairs`, `lookup_tables`)."""
import itertools

import numpy as np
import pytest

from oracle import semmoe_oracle as O


def _rand_instance(seed, E, D, U, dense=False):
    r = np.random.default_rng(seed)
    k = min(4, E)
    T = 40 * U
    ids = np.stack([r.choice(E, size=k, replace=False) for _ in range(T)]).astype(np.int32)
    load, coact = O.coact_hist(ids, E)
    unit_of = r.integers(0, U, size=T)
    act = O.token_expert_table(unit_of, ids, U, E)
    ln = np.bincount(unit_of, minlength=U)
    if dense:
        act = act + r.integers(0, 3, size=act.shape)
    return load, coact, act, ln, ids, unit_of


# ------------------------------------------------------------------ expert_place with the request term


@pytest.mark.parametrize("E,D,seed", [(8, 2, 0), (16, 4, 1), (12, 3, 2), (32, 8, 3)])
def test_without_the_request_term_it_is_place(E, D, seed):
    load, coact, act, ln, _, _ = _rand_instance(seed, E, D, 6)
    for alpha, gamma in [(1, 0), (3, 1), (1, 2)]:
        want = O.place(load, coact, D, alpha, gamma, 8)[0]
        ur = np.random.default_rng(seed).integers(0, D, size=6)
        got = O.expert_place_affinity(load, coact, D, act, ur, alpha, 0, gamma, 8)
        assert got.tolist() == want.tolist()
        got = O.expert_place_affinity(load, coact, D, None, None, alpha, 5, gamma, 8)
        assert got.tolist() == want.tolist()
        phys, inv = O.placement_order(got, D)
        assert phys.tolist() == O.place(load, coact, D, alpha, gamma, 8)[1].tolist()
        assert inv.tolist() == O.place(load, coact, D, alpha, gamma, 8)[2].tolist()


def test_request_term_alone_recovers_the_units_experts():
    """no co-activation information at all; units 0,1 (on cluster 0) activate {0,3,5,6}, units 2,3 (on cluster 1)
    activate {1,2,4,7}: every expert must follow the units that activate it"""
    E, D = 8, 2
    act = np.zeros((4, E), dtype=np.int64)
    for u in (0, 1):
        act[u, [0, 3, 5, 6]] = [4, 3, 2, 1]
    for u in (2, 3):
        act[u, [1, 2, 4, 7]] = [1, 2, 3, 4]
    load = act.sum(axis=0)
    coact = np.zeros((E, E), dtype=np.int64)
    got = O.expert_place_affinity(load, coact, D, act, [0, 0, 1, 1], alpha_e=1, beta_e=1, ft_passes=0)
    assert got.tolist() == [0, 1, 1, 0, 1, 0, 0, 1]
    # the units the other way round: the experts follow
    got = O.expert_place_affinity(load, coact, D, act, [1, 1, 0, 0], alpha_e=1, beta_e=1, ft_passes=0)
    assert got.tolist() == [1, 0, 0, 1, 0, 1, 1, 0]


def test_hand_example_of_the_three_terms():
    """E = 4, D = 2, loads 10, 9, 2, 1, coact(0,1) = 5, coact(2,3) = 1, one unit on cluster 1 with mass 7 on
    expert 1, one unit on cluster 0 with mass 1 on expert 2.  Expert 0 -> cluster 0 (all scores 0, equal loads,
    smaller c).  Expert 1 on (c0, c1): EAfE = (5, 0), EAfR = (0, 7), loads_cls = (10, 0):
      alpha 1, beta 0, gamma 0: (5, 0)   -> c0        alpha 1, beta 1, gamma 0: (5, 7)   -> c1
      alpha 1, beta 0, gamma 1: (-5, 0)  -> c1        alpha 2, beta 1, gamma 0: (10, 7)  -> c0"""
    load = np.array([10, 9, 2, 1])
    coact = np.zeros((4, 4), dtype=np.int64)
    coact[0, 1] = coact[1, 0] = 5
    coact[2, 3] = coact[3, 2] = 1
    act = np.array([[0, 7, 0, 0], [0, 0, 1, 0]])
    ur = [1, 0]
    f = lambda a, b, g: int(O.expert_place_affinity(load, coact, 2, act, ur, a, b, g, 0)[1])
    assert f(1, 0, 0) == 0
    assert f(1, 1, 0) == 1
    assert f(1, 0, 1) == 1
    assert f(2, 1, 0) == 0


def test_fine_tuning_swaps_on_the_weighted_gain():
    """greedy result {0,1 | 2,3} by co-activation; the units want {0,2 | 1,3}.  Swapping 1 and 2 loses
    coact(0,1)+coact(2,3) = 2 + 2 and gains the local mass R[1][c1] + R[2][c0] = 3 + 3: gain = -4*alpha + 6*beta.
    The greedy pass itself is run with beta = 0 by giving the units no mass on the first two experts placed."""
    load = np.array([4, 3, 2, 1])
    coact = np.zeros((4, 4), dtype=np.int64)
    coact[0, 1] = coact[1, 0] = 2
    coact[2, 3] = coact[3, 2] = 2
    act = np.array([[0, 0, 3, 0], [0, 3, 0, 0]])     # unit 0 on c0 wants expert 2, unit 1 on c1 wants expert 1
    ur = [0, 1]
    # greedy: e0 -> c0; e1: (2a + 0b, 0a + 3b); with a = 2, b = 1: 4 > 3 -> c0; e2, e3 -> c1 (c0 full)
    assert O.expert_place_affinity(load, coact, 2, act, ur, 2, 1, 0, 0).tolist() == [0, 0, 1, 1]
    # one sweep: pair (0,2): gain = a*(0+0-2-2) + b*(0 + 3 - 0 - 0) = -8 + 3 < 0; pair (0,3): -8 + 0 < 0;
    # pair (1,2): a*(-4) + b*(3 + 3) = -8 + 6 < 0  -> nothing moves (the other pairs lose more)
    assert O.expert_place_affinity(load, coact, 2, act, ur, 2, 1, 0, 4).tolist() == [0, 0, 1, 1]
    # a = 7, b = 4: greedy e1: (14, 12) -> c0; sweep pair (1,2): 7*(-4) + 4*6 = -4 < 0: stays
    assert O.expert_place_affinity(load, coact, 2, act, ur, 7, 4, 0, 4).tolist() == [0, 0, 1, 1]
    # unit 0's mass on expert 2 raised to 4, a = 5, b = 3:
    act2 = np.array([[0, 0, 4, 0], [0, 3, 0, 0]])
    # greedy e1: (10, 9) -> c0; sweep pair (0,2): 5*(-4) + 3*4 = -8; (0,3): -20; (1,2): 5*(-4) + 3*(3+4) = +1 -> swap
    assert O.expert_place_affinity(load, coact, 2, act2, ur, 5, 3, 0, 0).tolist() == [0, 0, 1, 1]
    assert O.expert_place_affinity(load, coact, 2, act2, ur, 5, 3, 0, 1).tolist() == [0, 1, 0, 1]


# ------------------------------------------------------------------ req_sched


def test_unit_schedule_hand_example():
    """U = 3, E = 2, D = 2 (two units per cluster at most), expert e on cluster e, unit_act rows (2,0), (1,1), (0,3),
    lengths 5, 4, 3 -> order u0, u1, u2.
    alpha_r = 1, beta_r = 10: u0: RAfR (0,0), RAfE (2,0) -> c0.  u1: RAfR (2*1+0*1, 0) = (2,0), RAfE (1,1):
      scores (12, 10) -> c0, now full.  u2 -> c1.
    alpha_r = 0: u1 scores (10, 10) equal -> the cluster with fewer tokens: c1; u2: RAfE (0,3) -> c1."""
    act = np.array([[2, 0], [1, 1], [0, 3]])
    ln = [5, 4, 3]
    assert O.unit_schedule(act, ln, [0, 1], 2, alpha_r=1, beta_r=10).tolist() == [0, 0, 1]
    assert O.unit_schedule(act, ln, [0, 1], 2, alpha_r=0, beta_r=10).tolist() == [0, 1, 1]
    # longest first: with lengths reversed u2 picks first and the equal-score unit sees tokens on c1
    assert O.unit_schedule(act, [3, 4, 5], [0, 1], 2, alpha_r=0, beta_r=10).tolist() == [0, 0, 1]


@pytest.mark.parametrize("E,D,seed", [(16, 4, 0), (32, 8, 1), (8, 2, 2)])
def test_unit_schedule_is_the_mass_argmax_when_no_cluster_fills(E, D, seed):
    """request-expert term alone and exactly U/D units preferring every cluster: every unit gets the cluster
    holding most of its activation mass, which is what `lookup_tables` (pinned elsewhere) calls dev"""
    r = np.random.default_rng(seed)
    e2r = r.permutation(np.repeat(np.arange(D), E // D))
    per = 3
    U = per * D
    act = np.zeros((U, E), dtype=np.int64)
    want = np.repeat(np.arange(D), per)
    r.shuffle(want)
    for u in range(U):
        act[u] = r.integers(0, 3, size=E)
        act[u, np.flatnonzero(e2r == want[u])] += 20
    ln = r.integers(1, 100, size=U)
    dev, _, _ = O.lookup_tables(act, e2r, D, 4)
    assert dev.tolist() == want.tolist()
    assert O.unit_schedule(act, ln, e2r, D, 0, 1).tolist() == want.tolist()


def test_request_request_term_groups_units_of_equal_support():
    """alpha_r only: units with disjoint supports have RAfR = 0 towards each other, so the second support opens
    the emptier cluster and its peers follow it, whatever the placement says"""
    act = np.array([[5, 5, 0, 0], [0, 0, 4, 4], [3, 3, 0, 0], [0, 0, 2, 2]])
    ln = [10, 8, 6, 4]
    e2r = [0, 1, 0, 1]          # placement splits both supports: it must not matter
    assert O.unit_schedule(act, ln, e2r, 2, alpha_r=1, beta_r=0).tolist() == [0, 1, 0, 1]


@pytest.mark.parametrize("U,D", [(7, 3), (10, 4), (5, 5), (3, 8)])
def test_unit_schedule_respects_the_unit_cap(U, D):
    r = np.random.default_rng(U * 31 + D)
    act = r.integers(0, 5, size=(U, 8 * D))
    act[:, :8] += 50           # every unit prefers cluster 0
    e2r = np.repeat(np.arange(D), 8)
    ur = O.unit_schedule(act, r.integers(1, 9, size=U), e2r, D, 1, 1)
    assert np.bincount(ur, minlength=D).max() <= -(-U // D)
    assert np.bincount(ur, minlength=D)[0] == -(-U // D)


# ------------------------------------------------------------------ score


def test_score_hand_example():
    """rows (2,0), (1,1), (0,3), units on (0,0,1), expert e on cluster e, lengths 5,4,3: tokens (9,3) -> 9;
    remote mass: unit 1's activation of expert 1 only -> 1"""
    act = np.array([[2, 0], [1, 1], [0, 3]])
    assert O.coschedule_score(act, [5, 4, 3], [0, 1], [0, 0, 1], 2, 1, 2) == (11, 9, 1)
    assert O.coschedule_score(act, [5, 4, 3], [1, 0], [0, 0, 1], 2, 3, 1) == (3 * 9 + 6, 9, 6)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_remote_mass_is_the_remote_pair_count_when_every_token_is_a_unit(seed):
    r = np.random.default_rng(seed)
    E, D, k, T = 16, 4, 3, 60
    ids = np.stack([r.choice(E, size=k, replace=False) for _ in range(T)]).astype(np.int32)
    e2r = r.permutation(np.repeat(np.arange(D), E // D))
    tr = r.integers(0, D, size=T)
    act = O.token_expert_table(np.arange(T), ids, T, E)
    sc, mx, remote = O.coschedule_score(act, np.ones(T, dtype=int), e2r, tr, D, 1, 1)
    assert remote == T * k - O.local_pairs(ids, e2r, tr)
    assert mx == np.bincount(tr, minlength=D).max()


# ------------------------------------------------------------------ the alternation


def _planted(seed, D, m, per, noise):
    """D topics of m experts (ids scrambled) and `per` units per topic; a unit's tokens activate its topic's experts,
    a fraction `noise` of them anything"""
    r = np.random.default_rng(seed)
    E, U = D * m, D * per
    perm = r.permutation(E)
    topic_of_unit = np.repeat(np.arange(D), per)
    r.shuffle(topic_of_unit)
    k = 2
    ids, unit_of = [], []
    for u in range(U):
        for _ in range(int(r.integers(20, 40))):
            if r.random() < noise:
                row = r.choice(E, size=k, replace=False)
            else:
                row = perm[topic_of_unit[u] * m + r.choice(m, size=k, replace=False)]
            ids.append(row)
            unit_of.append(u)
    ids = np.array(ids, dtype=np.int32)
    unit_of = np.array(unit_of)
    load, coact = O.coact_hist(ids, E)
    act = O.token_expert_table(unit_of, ids, U, E)
    return load, coact, act, np.bincount(unit_of, minlength=U), topic_of_unit, perm


@pytest.mark.parametrize("seed,D,m,per", [(0, 2, 4, 3), (1, 4, 4, 2), (2, 4, 2, 4)])
def test_planted_topics_are_recovered(seed, D, m, per):
    load, coact, act, ln, topic, perm = _planted(seed, D, m, per, noise=0.0)
    e2r, ur, scores, best = O.coschedule(load, coact, act, ln, D, 1, 1, 0, 0, 1, 4, 3, 0, 1)
    assert scores[best] == 0                                   # nothing remote
    for t in range(D):
        cl = set(ur[topic == t].tolist())
        assert len(cl) == 1                                    # a topic's units share a cluster
        assert set(e2r[perm[t * m:(t + 1) * m]].tolist()) == cl   # and its experts sit there


def test_misleading_coactivation_is_overruled_by_the_request_term():
    """co-activation (from another workload) ties experts 0-1 and 2-3 together; the units at hand activate {0,2}
    or {1,3}.  With beta_e = 0 the placement follows the co-activation and half of the mass is remote whatever the
    units do; with the request term weighted in, the alternation reaches zero remote mass."""
    load = np.array([8, 8, 8, 8])
    coact = np.zeros((4, 4), dtype=np.int64)
    coact[0, 1] = coact[1, 0] = 3
    coact[2, 3] = coact[3, 2] = 3
    act = np.array([[6, 0, 6, 0], [0, 5, 0, 5], [4, 0, 4, 0], [0, 3, 0, 3]])
    ln = [12, 10, 8, 6]
    e2r, ur, scores, best = O.coschedule(load, coact, act, ln, 2, 1, 0, 0, 0, 1, 4, 3, 0, 1)
    assert e2r.tolist() == [0, 0, 1, 1] and scores[best] == 18
    e2r, ur, scores, best = O.coschedule(load, coact, act, ln, 2, 1, 1, 0, 1, 1, 4, 3, 0, 1)
    assert scores[best] == 0
    assert e2r[0] == e2r[2] != e2r[1] == e2r[3]


def _all_balanced(n, D):
    """all assignments of n items to D clusters with at most ceil(n/D) per cluster"""
    cap = -(-n // D)
    for a in itertools.product(range(D), repeat=n):
        if max(np.bincount(a, minlength=D)) <= cap:
            yield a


@pytest.mark.parametrize("seed", range(6))
def test_never_below_the_brute_force_optimum_and_step_bookkeeping(seed):
    E, D, U = 4, 2, 4
    load, coact, act, ln, _, _ = _rand_instance(seed, E, D, U, dense=True)
    w_load, w_comm = 2, 1
    e2r, ur, scores, best = O.coschedule(load, coact, act, ln, D, 1, 1, 0, 1, 1, 4, 3, w_load, w_comm)
    assert len(scores) == 3 and scores[best] == min(scores) and best == scores.index(min(scores))
    assert O.coschedule_score(act, ln, e2r, ur, D, w_load, w_comm)[0] == scores[best]
    assert np.bincount(e2r, minlength=D).tolist() == [E // D] * D
    assert np.bincount(ur, minlength=D).max() <= -(-U // D)
    opt = min(O.coschedule_score(act, ln, pe, pu, D, w_load, w_comm)[0]
              for pe in _all_balanced(E, D) if np.bincount(pe, minlength=D).min() == E // D
              for pu in _all_balanced(U, D))
    assert scores[best] >= opt


def test_one_step_is_place_then_schedule_then_place_then_schedule():
    load, coact, act, ln, _, _ = _rand_instance(5, 16, 4, 9)
    e0 = O.place(load, coact, 4, 2, 1, 3)[0]
    u0 = O.unit_schedule(act, ln, e0, 4, 1, 2)
    e1 = O.expert_place_affinity(load, coact, 4, act, u0, 2, 3, 1, 3)
    u1 = O.unit_schedule(act, ln, e1, 4, 1, 2)
    e2r, ur, scores, best = O.coschedule(load, coact, act, ln, 4, 2, 3, 1, 1, 2, 3, 1, 1, 1)
    assert best == 0 and e2r.tolist() == e1.tolist() and ur.tolist() == u1.tolist()


# ------------------------------------------------------------------ token labels


def test_token_labels_hand_example():
    """requests [0,1,1], [1,2], [1,0,3] on clusters 1, 0, 1; V = 5, k = 4.
    id 0: counts (0,2) -> 1, share 1.  id 1: (1,3) -> 1, share 3/4 -> 49152, level 3.  id 2: (1,0) -> 0.
    id 3: (0,1) -> 1.  id 4 never occurs."""
    off = np.array([0, 3, 5, 8])
    keys = np.array([0, 1, 1, 1, 2, 1, 0, 3])
    dev, conf, level = O.token_labels(off, keys, [1, 0, 1], 5, 2, 4)
    assert dev.tolist() == [1, 1, 0, 1, -1]
    assert conf.tolist() == [65536, 49152, 65536, 65536, 0]
    assert level.tolist() == [4, 3, 4, 4, 0]


@pytest.mark.parametrize("seed,D", [(0, 2), (1, 4), (2, 8)])
def test_token_labels_are_lookup_tables_of_the_count_table(seed, D):
    """the count table [V, D] read as an activation table over D 'experts', expert c on cluster c"""
    r = np.random.default_rng(seed)
    V, n_req, k = 30, 12, 6
    lens = r.integers(1, 40, size=n_req)
    off = np.concatenate([[0], np.cumsum(lens)])
    keys = r.integers(0, V - 3, size=off[-1])           # the last three ids never occur
    req_rank = r.integers(0, D, size=n_req)
    tok_rank = np.repeat(req_rank, lens)
    table = np.zeros((V, D), dtype=np.int64)
    np.add.at(table, (keys, tok_rank), 1)
    want = O.lookup_tables(table, np.arange(D), D, k)
    got = O.token_labels(off, keys, req_rank, V, D, k)
    for a, b in zip(got, want):
        assert a.tolist() == b.tolist()
