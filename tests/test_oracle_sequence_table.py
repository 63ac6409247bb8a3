"""Pins of the oracle's inter-layer device-sequence table (App. B: the rows of the table are the devices selected
at the previous layers) and of Alg. 3's `cond(T_p > A_p, T, A)` with both tables: hand examples, the special cases
that are functions pinned elsewhere (`gain_matrix`, `reshuffle_lookup`), the strictness of the comparison."""
import numpy as np
import pytest

from oracle import semmoe_oracle as O


def test_device_sequence_hand_example():
    """experts 0-1 on device 0, 2-3 on device 1, 4-5 on device 2.  k = 3.
    token 0: experts 0,1,4 -> counts (2,0,1) -> 0;  token 1: 2,4,5 -> (0,1,2) -> 2;  token 2: 0,2,4 -> (1,1,1) -> 0
    (equal -> smallest);  token 3: 3,5,2 -> (0,2,1) -> 1"""
    e2r = [0, 0, 1, 1, 2, 2]
    ids = np.array([[0, 1, 4], [2, 4, 5], [0, 2, 4], [3, 5, 2]])
    assert O.device_sequence(ids, e2r, 3).tolist() == [0, 2, 0, 1]
    # chained: previous sequence numbers 2, 0, -1 (unknown), 1 -> 2*3+0, 0*3+2, unknown, 1*3+1
    assert O.device_sequence(ids, e2r, 3, [2, 0, -1, 1]).tolist() == [6, 2, -1, 4]
    # two layers back then one layer back: the older layer is the more significant digit
    older = O.device_sequence(ids[::-1], e2r, 3)                 # devices 1, 0, 2, 0
    assert O.device_sequence(ids, e2r, 3, older).tolist() == [3, 2, 6, 1]


@pytest.mark.parametrize("E,D,k,seed", [(16, 4, 2, 0), (64, 8, 8, 1), (12, 3, 5, 2), (8, 8, 3, 3)])
def test_device_is_the_first_argmax_of_the_gain_matrix(E, D, k, seed):
    r = np.random.default_rng(seed)
    ids = np.stack([r.choice(E, size=k, replace=False) for _ in range(300)])
    e2r = r.permutation(np.repeat(np.arange(D), E // D))
    want = O.gain_matrix(ids, e2r, D).argmax(axis=1)
    assert O.device_sequence(ids, e2r, D).tolist() == want.tolist()
    prev = r.integers(-1, D * D, size=300)
    got = O.device_sequence(ids, e2r, D, prev)
    assert got.tolist() == np.where(prev < 0, -1, prev * D + want).tolist()


def test_sequence_table_rows_are_the_activation_table_keyed_by_the_sequence():
    """two tokens with history (1, 0) activate devices' experts: the row of sequence number 1*D+0 collects them"""
    D, E = 2, 4
    e2r = [0, 0, 1, 1]
    seq = np.array([2, 2, 1, -1])
    ids = np.array([[0, 2], [0, 1], [3, 2], [1, 0]])
    table = O.token_expert_table(seq[seq >= 0], ids[seq >= 0], D * D, E)
    assert table[2].tolist() == [2, 1, 1, 0] and table[1].tolist() == [0, 0, 1, 1] and table[0].sum() == 0
    dev_a, conf_a, level_a = O.lookup_tables(table, e2r, D, 2)
    assert dev_a.tolist() == [-1, 1, 0, -1]
    assert conf_a.tolist() == [0, 65536, 49152, 0]       # row 2: 3 of 4 activations on device 0


def _tables(r, V, D, k, unseen):
    dev = r.integers(0, D, size=V).astype(np.int32)
    conf = r.integers(0, 65537, size=V).astype(np.int32)
    level = ((2 * k * conf.astype(np.int64) + 65536) // (2 * 65536)).astype(np.int32)
    gone = r.random(V) < unseen
    dev[gone], conf[gone], level[gone] = -1, 0, 0
    return dev, conf, level


def test_cond_hand_example():
    """D = 2, 4 tokens, cap 2, homes 0,0,1,1; k = 4.
    token 0: T (dev 1, conf 40000, level 2), A (dev 0, conf 50000, level 3): T_p > A_p false -> A: device 0
    token 1: T (1, 50000, 3), A (0, 40000, 2) -> T: device 1
    token 2: T (0, 30000, 2), A (1, 30000, 1): equal -> not greater -> A: device 1
    token 3: T unseen, A index outside its table -> home 1, priority 0
    preferences (0, 1, 1, 1): rank 1 is asked by tokens 1 (level 3), 2 (level 1), 3 (0) -> keeps 1, 2; token 3 spills to 0"""
    dev, conf, level = np.array([1, 1, 0, -1]), np.array([40000, 50000, 30000, 0]), np.array([2, 3, 2, 0])
    dev_a, conf_a, level_a = np.array([0, 0, 1]), np.array([50000, 40000, 30000]), np.array([3, 2, 1])
    keys, seq = np.array([0, 1, 2, 3]), np.array([0, 1, 2, 7])
    tr, shf, inv, rc = O.reshuffle_cond(keys, dev, conf, level, seq, dev_a, conf_a, level_a, -1, 2, 2)
    assert tr.tolist() == [0, 1, 1, 0] and rc.tolist() == [2, 2]
    assert shf.tolist() == [0, 3, 1, 2] and inv[shf].tolist() == [0, 1, 2, 3]
    # a threshold of 45000 leaves only the entries above it: token 0 (A, 50000) and token 1 (T, 50000); 2 and 3 stay
    # home: preferences (0, 1, 1, 1) with priorities (3, 3, 0, 0): rank 1 keeps tokens 1 and 2, token 3 spills
    tr, _, _, _ = O.reshuffle_cond(keys, dev, conf, level, seq, dev_a, conf_a, level_a, 45000, 2, 2)
    assert tr.tolist() == [0, 1, 1, 0]
    # with room for three, token 3 stays at home as well
    tr, _, _, _ = O.reshuffle_cond(keys, dev, conf, level, seq, dev_a, conf_a, level_a, 45000, 2, 3)
    assert tr.tolist() == [0, 1, 1, 1]
    # "exceeds": a confidence equal to the threshold is not followed -> everybody home
    tr, _, _, _ = O.reshuffle_cond(keys, dev, conf, level, seq, dev_a, conf_a, level_a, 50000, 2, 2)
    assert tr.tolist() == [0, 0, 1, 1]
    tr, _, _, _ = O.reshuffle_cond(keys, dev, conf, level, seq, dev_a, conf_a, level_a, 49999, 2, 2)
    assert tr.tolist() == [0, 1, 1, 0]
    # a token with no entry in either table stays home whatever the threshold
    tr, _, _, _ = O.reshuffle_cond(keys, dev, conf, level, seq, dev_a, conf_a, level_a, -5, 2, 3)
    assert tr.tolist() == [0, 1, 1, 1]


@pytest.mark.parametrize("T,V,D,k,thr,seed", [(300, 40, 4, 2, -1, 0), (500, 64, 8, 8, 20000, 1), (257, 16, 3, 4, 0, 2)])
def test_cond_without_a_sequence_table_is_the_rebatch_from_the_schedule_table(T, V, D, k, thr, seed):
    r = np.random.default_rng(seed)
    dev, conf, level = _tables(r, V, D, k, 0.2)
    keys = r.integers(0, V, size=T)
    cap = -(-T // D)
    want = O.reshuffle_lookup(keys, dev, conf, level, thr, D, cap)
    none = (np.full(4, -1), np.zeros(4, dtype=int), np.zeros(4, dtype=int))
    got = O.reshuffle_cond(keys, dev, conf, level, r.integers(-1, 6, size=T), *none, thr, D, cap)
    for a, b in zip(got, want):
        assert a.tolist() == b.tolist()
    # and the other way round: no schedule table, the sequence table alone
    got = O.reshuffle_cond(r.integers(-1, 6, size=T), *none, keys, dev, conf, level, thr, D, cap)
    for a, b in zip(got, want):
        assert a.tolist() == b.tolist()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cond_takes_per_token_the_table_of_higher_confidence(seed):
    """capacity never binds (cap = T): every token lands where the chosen entry says"""
    r = np.random.default_rng(seed)
    T, V, VA, D, k = 400, 50, 16, 4, 4
    dev, conf, level = _tables(r, V, D, k, 0.1)
    dev_a, conf_a, level_a = _tables(r, VA, D, k, 0.1)
    keys, seq = r.integers(0, V, size=T), r.integers(-1, VA, size=T)
    tr, _, _, _ = O.reshuffle_cond(keys, dev, conf, level, seq, dev_a, conf_a, level_a, -1, D, T)
    home = O.home_rank(T, D)
    for i in range(T):
        ct = conf[keys[i]] if dev[keys[i]] >= 0 else -1
        ca = conf_a[seq[i]] if seq[i] >= 0 and dev_a[seq[i]] >= 0 else -1
        want = dev[keys[i]] if ct > ca else (dev_a[seq[i]] if ca >= 0 else home[i])
        assert tr[i] == want, i
