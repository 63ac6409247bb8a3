"""Pins of the oracle's request scheduling (Alg. 2 `get_dp_rank` / `schedule`, Attention-DP scenario) against what
the paper and the mathematics fix: a hand-worked example, the request-to-cluster rule S_r of Sec. 3.3 where the mask
cannot interfere, the guarantee that any D consecutive requests of a round reach all D ranks, and degenerate cases."""
import numpy as np
import pytest

from oracle import semmoe_oracle as O
import workloads as WL


def _offsets(lens):
    off = np.zeros(len(lens) + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    return off


def test_hand_example_with_mask_and_reset():
    """D = 2, keys 0,1 -> device 1, key 2 -> device 0, key 3 never profiled.
    r0 = [0,1,2]   scores (1,2) -> device 1; mask {1}
    r1 = [0,0,0,1] scores (0,4) -> device 1 is masked -> device 0; every device masked -> reset
    r2 = [2,3,3]   scores (1,0) -> device 0; mask {0}
    r3 = [2,2]     scores (2,0) -> device 0 masked -> device 1; reset
    r4 = [3]       scores (0,0) -> equal -> the smallest id, device 0"""
    dev = np.array([1, 1, 0, -1], dtype=np.int32)
    keys = np.array([0, 1, 2, 0, 0, 0, 1, 2, 3, 3, 2, 2, 3], dtype=np.int32)
    off = _offsets([3, 4, 3, 2, 1])
    assert O.request_schedule(off, keys, dev, 2).tolist() == [1, 0, 0, 1, 0]
    tr, shf, inv, rc = O.request_assignment(off, [1, 0, 0, 1, 0], 2)
    assert tr.tolist() == [1, 1, 1, 0, 0, 0, 0, 0, 0, 0, 1, 1, 0]
    assert shf.tolist() == [3, 4, 5, 6, 7, 8, 9, 12, 0, 1, 2, 10, 11]
    assert rc.tolist() == [8, 5]
    assert (inv[shf] == np.arange(13)).all()


@pytest.mark.parametrize("D,seed", [(4, 0), (8, 1), (16, 2)])
def test_equals_the_request_to_cluster_rule_when_argmaxes_are_distinct(D, seed):
    """within one round, requests whose best devices are all different each get S_r = argmax_j sum_i R_ij
    (here computed with bincount over the looked-up devices): the mask never bites"""
    r = np.random.default_rng(seed)
    V = 50
    dev = r.integers(0, D, size=V).astype(np.int32)
    targets = r.permutation(D)
    lens, keys = [], []
    for q in range(D):
        ln = int(r.integers(5, 30))
        strong = r.choice(np.flatnonzero(dev == targets[q]), size=ln) if (dev == targets[q]).any() else None
        if strong is None:
            pytest.skip("a device without keys")
        noise = r.integers(0, V, size=ln // 3)
        kk = np.concatenate([strong, noise])
        lens.append(len(kk))
        keys.append(kk)
    keys = np.concatenate(keys).astype(np.int32)
    off = _offsets(lens)
    want = [int(np.bincount(dev[keys[off[q]:off[q + 1]]], minlength=D).argmax()) for q in range(D)]
    assert sorted(want) == list(range(D))
    assert O.request_schedule(off, keys, dev, D).tolist() == want


@pytest.mark.parametrize("D,n_req,seed", [(4, 23, 0), (8, 64, 1), (3, 10, 2), (32, 100, 3), (1, 5, 4)])
def test_every_round_reaches_every_rank(D, n_req, seed):
    """continual D requests are distributed to all D ranks (Sec. 3.3): every aligned window of D requests is a
    permutation of the ranks, so request counts per rank differ by at most one"""
    r = np.random.default_rng(seed)
    V = 40
    dev = r.integers(-1, D, size=V).astype(np.int32)
    lens = r.integers(0, 20, size=n_req)
    keys = r.integers(0, V, size=int(lens.sum())).astype(np.int32)
    rr = O.request_schedule(_offsets(lens), keys, dev, D)
    for s in range(0, n_req - D + 1, D):
        assert sorted(rr[s:s + D].tolist()) == list(range(D))
    cnt = np.bincount(rr, minlength=D)
    assert cnt.max() - cnt.min() <= 1
    # the first request of every round sees no mask: it gets its global best device
    off = _offsets(lens)
    for s in range(0, n_req, D):
        d = dev[keys[off[s]:off[s + 1]]]
        sc = np.bincount(d[d >= 0], minlength=D)
        assert rr[s] == int(sc.argmax())


def test_masked_choice_is_the_best_of_what_is_left():
    """brute force over the unmasked set, request by request, on a small case"""
    r = np.random.default_rng(9)
    D, V, n_req = 5, 30, 17
    dev = r.integers(0, D, size=V).astype(np.int32)
    lens = r.integers(1, 12, size=n_req)
    keys = r.integers(0, V, size=int(lens.sum())).astype(np.int32)
    off = _offsets(lens)
    rr = O.request_schedule(off, keys, dev, D)
    used = set()
    for q in range(n_req):
        sc = np.bincount(dev[keys[off[q]:off[q + 1]]], minlength=D)
        left = [x for x in range(D) if x not in used]
        top = max(sc[x] for x in left)
        assert rr[q] == min(x for x in left if sc[x] == top)
        used.add(int(rr[q]))
        if len(used) == D:
            used = set()


def test_unseen_keys_give_round_robin_and_one_rank_gives_zero():
    dev = np.full(8, -1, dtype=np.int32)
    off = _offsets([3, 1, 4, 1, 5, 9, 2])
    keys = np.arange(25, dtype=np.int32) % 8
    assert O.request_schedule(off, keys, dev, 3).tolist() == [0, 1, 2, 0, 1, 2, 0]
    assert O.request_schedule(off, keys, np.zeros(8, dtype=np.int32), 1).tolist() == [0] * 7


def test_assignment_is_the_stable_sort_by_request_rank():
    r = np.random.default_rng(3)
    D = 6
    lens = r.integers(0, 15, size=40)
    off = _offsets(lens)
    rr = r.integers(0, D, size=40)
    tr, shf, inv, rc = O.request_assignment(off, rr, D)
    T = int(off[-1])
    assert (tr == np.repeat(rr, lens)).all()
    assert sorted(shf.tolist()) == list(range(T)) and (inv[shf] == np.arange(T)).all()
    assert (np.diff(tr[shf]) >= 0).all()
    for x in range(D):                                  # a rank holds its tokens in arrival order
        assert (np.diff(shf[tr[shf] == x]) > 0).all()
        assert rc[x] == lens[rr == x].sum()


def test_requests_of_one_topic_follow_the_topic_rank_on_the_synthetic_workload():
    """on the request workload (runs of tokens of one topic) the scheduled rank of a round's first request is the
    rank that holds most of the topic's cluster: the table-driven request rule recovers the planted semantics"""
    w = WL.CONFIGS["c2_qwen3_30b"]
    off, cls, keys = WL.requests(w, profile=True, n=4096)
    assert off[0] == 0 and off[-1] == 4096 and (np.diff(off) > 0).all()
    assert keys.min() >= 0 and keys.max() < WL.vocab_size(w)
    # a schedule table that knows the classes: key of class c -> rank c % D
    V = WL.vocab_size(w)
    dev = ((np.arange(V) // WL.KEYS_PER_CLASS) % w.D).astype(np.int32)
    dev[w.C * WL.KEYS_PER_CLASS:] = -1
    rr = O.request_schedule(off, keys, dev, w.D)
    for s in range(0, len(off) - 1, w.D):
        c = np.bincount(cls[off[s]:off[s + 1]][cls[off[s]:off[s + 1]] >= 0], minlength=w.C)
        byrank = np.bincount(np.arange(w.C) % w.D, weights=c, minlength=w.D)
        assert rr[s] == int(byrank.argmax())
