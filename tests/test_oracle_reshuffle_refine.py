"""Pins of the oracle's `reshuffle_refine` (greedy rebatch of Alg. 3, then moves of placed tokens until the
communication term of the Sec. 3.3 objective is minimal): hand examples of a swap between two ranks and of a move
into free room, the optimum of the min-cost flow and of brute force, validity, and the budget of cycles."""
import numpy as np
import pytest

from oracle import semmoe_oracle as O
import workloads as WL


def _valid(ids, e2r, D, cap, out):
    tr, shf, inv, cnt = out
    T = ids.shape[0]
    assert tr.min() >= 0 and tr.max() < D
    assert (np.bincount(tr, minlength=D) == cnt).all() and cnt.max() <= cap and cnt.sum() == T
    assert (shf == np.argsort(tr, kind="stable")).all()
    assert (inv[shf] == np.arange(T)).all()


def test_refine_hand_example_swap_between_two_ranks():
    # D = 4, cap = 1, three experts per rank (rank r: experts 3r .. 3r+2), home = [0, 1, 2, 3]
    e2r = np.repeat(np.arange(4), 3)
    ids = np.array([[0, 1, 9],    # g = (2,0,0,1): proposes rank 0 with 2
                    [3, 4, 6],    # g = (0,2,1,0): proposes rank 1 with 2
                    [0, 1, 2],    # g = (3,0,0,0): proposes rank 0 with 3 -> kept there
                    [3, 4, 5]])   # g = (0,3,0,0): proposes rank 1 with 3 -> kept there
    # greedy: tokens 0 and 1 lose their ranks and take the free slots in rank order: token 0 -> rank 2 (gain 0),
    # token 1 -> rank 3 (gain 0): 6 local pairs
    g0 = O.reshuffle(ids, e2r, 4, 1)[0]
    assert list(g0) == [2, 3, 0, 1] and O.local_pairs(ids, e2r, g0) == 6
    # residual arcs 2 -> 3 (token 0: 1 - 0) and 3 -> 2 (token 1: 1 - 0): a closed walk of gain 2, one cycle
    out, cycles, conv = O.reshuffle_refine(ids, e2r, 4, 1)
    assert list(out[0]) == [3, 2, 0, 1] and cycles == 1 and conv
    assert O.local_pairs(ids, e2r, out[0]) == 8 == O.reshuffle_bruteforce(ids, e2r, 4, 1)
    _valid(ids, e2r, 4, 1, out)


def test_refine_hand_example_move_into_free_room():
    # D = 3, cap = 2, T = 4 (two slots stay free), two experts per rank, home = [0, 0, 1, 1]
    e2r = np.repeat(np.arange(3), 2)
    ids = np.array([[0, 1],    # g = (2,0,0)
                    [0, 1],    # g = (2,0,0)
                    [0, 4],    # g = (1,0,1): home 1 is no maximiser -> proposes rank 0 with 1, loses to tokens 0, 1
                    [2, 3]])   # g = (0,2,0)
    # greedy: token 2 takes the first free slot, on rank 1 (gain 0)
    g0 = O.reshuffle(ids, e2r, 3, 2)[0]
    assert list(g0) == [0, 0, 1, 1] and O.local_pairs(ids, e2r, g0) == 6
    # rank 2 has room: the walk Z -> 1 -> 2 -> Z gains 1 (token 2: g[2] - g[1])
    out, cycles, conv = O.reshuffle_refine(ids, e2r, 3, 2)
    assert list(out[0]) == [0, 0, 2, 1] and cycles == 1 and conv
    assert O.local_pairs(ids, e2r, out[0]) == 7 == O.reshuffle_bruteforce(ids, e2r, 3, 2)
    _valid(ids, e2r, 3, 2, out)


def test_refine_rotation_over_three_ranks_where_no_exchange_of_two_gains():
    e2r = np.array([0, 1, 2])
    ids = np.array([[0, 1, 1],    # g = (1,2,0), on rank 0: +1 to rank 1, -1 to rank 2
                    [1, 2, 2],    # g = (0,1,2), on rank 1: +1 to rank 2, -1 to rank 0
                    [2, 0, 0]])   # g = (2,0,1), on rank 2: +1 to rank 0, -1 to rank 1
    # every closed walk over two ranks gains 1 - 1 = 0; the rotation 0 -> 1 -> 2 -> 0 gains 3
    out, cycles, conv = O.reshuffle_refine(ids, e2r, 3, 1, start=[0, 1, 2])
    assert list(out[0]) == [1, 2, 0] and cycles == 1 and conv
    assert O.local_pairs(ids, e2r, out[0]) == 6 == O.reshuffle_bruteforce(ids, e2r, 3, 1)


def test_refine_which_walk_which_tokens_how_many():
    # two disjoint exchanges of equal gain: the walk through the smallest rank goes first
    e2r = np.array([0, 1, 2, 3])
    ids = np.array([[1], [0], [3], [2]])
    out, cycles, conv = O.reshuffle_refine(ids, e2r, 4, 1, max_cycles=1, start=[0, 1, 2, 3])
    assert list(out[0]) == [1, 0, 2, 3] and cycles == 1 and not conv
    out, cycles, conv = O.reshuffle_refine(ids, e2r, 4, 1, start=[0, 1, 2, 3])
    assert list(out[0]) == [1, 0, 3, 2] and cycles == 2 and conv
    # rank 0's token can exchange with rank 1's or rank 2's for the same gain: the walk back takes the smaller rank
    e2r = np.array([0, 1, 2])
    ids = np.array([[1, 2], [0, 0], [0, 0]])       # g = (0,1,1), (2,0,0), (2,0,0)
    out, cycles, conv = O.reshuffle_refine(ids, e2r, 3, 1, start=[0, 1, 2])
    assert list(out[0]) == [1, 0, 2] and cycles == 1 and conv
    # as many tokens per cycle as every arc of the walk has: two here, in one cycle
    e2r = np.array([0, 1])
    ids = np.array([[1], [1], [0], [0]])
    out, cycles, conv = O.reshuffle_refine(ids, e2r, 2, 2, start=[0, 0, 1, 1])
    assert list(out[0]) == [1, 1, 0, 0] and cycles == 1 and conv
    # three tokens of rank 0 want rank 1, one token comes back: one moves, the one of smallest index
    ids = np.array([[1], [1], [1], [0], [1], [1]])
    out, cycles, conv = O.reshuffle_refine(ids, e2r, 2, 3, start=[0, 0, 0, 1, 1, 1])
    assert list(out[0]) == [1, 0, 0, 0, 1, 1] and cycles == 1 and conv


def test_refine_free_room_bounds_the_number_of_movers():
    # D = 3, cap = 2, T = 5, home = [0,0,1,1,2]; tokens 2 and 3 lose rank 0 and are spilled onto rank 1; rank 2 has one
    # slot left, so only one of them (the smaller index) may follow its gain there
    e2r = np.repeat(np.arange(3), 2)
    ids = np.array([[0, 1], [0, 1], [0, 4], [0, 4], [4, 5]])
    g0 = O.reshuffle(ids, e2r, 3, 2)[0]
    assert list(g0) == [0, 0, 1, 1, 2]
    out, cycles, conv = O.reshuffle_refine(ids, e2r, 3, 2)
    assert list(out[0]) == [0, 0, 2, 1, 2] and cycles == 1 and conv
    _valid(ids, e2r, 3, 2, out)
    assert O.local_pairs(ids, e2r, out[0]) == 7 == O.reshuffle_bruteforce(ids, e2r, 3, 2)


def test_refine_after_spill_rounds_reaches_the_same_optimum_in_fewer_cycles():
    r = np.random.default_rng(11)
    T, E, D, k = 128, 32, 8, 4
    p = 1.0 / np.arange(1, E + 1) ** 1.2
    p /= p.sum()
    ids = np.stack([r.choice(E, size=k, replace=False, p=p) for _ in range(T)])
    e2r, _, _ = O.vanilla_placement(E, D)
    cap = T // D
    a, na, ca = O.reshuffle_refine(ids, e2r, D, cap)
    b, nb, cb = O.reshuffle_refine(ids, e2r, D, cap, rounds=3)
    assert ca and cb and O.local_pairs(ids, e2r, a[0]) == O.local_pairs(ids, e2r, b[0]) == O.reshuffle_exact(ids, e2r, D, cap)[1]
    assert nb <= na
    # no cycle allowed: the spill rounds themselves
    z, nz, cz = O.reshuffle_refine(ids, e2r, D, cap, 0, rounds=3)
    for x, y in zip(z, O.reshuffle_rounds(ids, e2r, D, cap, 3)):
        assert (x == y).all()


@pytest.mark.parametrize("seed", range(10))
def test_refine_reaches_the_bruteforce_optimum_on_tiny_inputs(seed):
    r = np.random.default_rng(900 + seed)
    T, D = int(r.integers(5, 9)), int(r.integers(2, 4))
    E, k = 2 * D, int(r.integers(1, 4))
    ids = WL.uniform_random_ids(T, E, min(k, E), seed=700 + seed)
    e2r, _, _ = O.vanilla_placement(E, D)
    cap = -(-T // D)
    out, cycles, conv = O.reshuffle_refine(ids, e2r, D, cap)
    assert conv
    _valid(ids, e2r, D, cap, out)
    assert O.local_pairs(ids, e2r, out[0]) == O.reshuffle_bruteforce(ids, e2r, D, cap)


@pytest.mark.parametrize("T,E,D,k,cf,skew", [(96, 16, 4, 2, 1.0, 1.2), (120, 32, 8, 4, 1.0, 1.1), (90, 18, 3, 3, 1.0, 1.5),
                                             (100, 16, 4, 3, 1.25, 1.3), (77, 24, 6, 2, 1.0, 1.0), (128, 32, 8, 8, 1.0, 1.2)])
def test_refine_equals_the_min_cost_flow_optimum_when_capacity_binds(T, E, D, k, cf, skew):
    # Zipf-skewed experts so that a few ranks are wanted by far more tokens than they can hold
    r = np.random.default_rng(T * 31 + E)
    p = 1.0 / np.arange(1, E + 1) ** skew
    p /= p.sum()
    ids = np.stack([r.choice(E, size=k, replace=False, p=p) for _ in range(T)])
    e2r, _, _ = O.vanilla_placement(E, D)
    cap = int(np.ceil(cf * T / D))
    greedy = O.local_pairs(ids, e2r, O.reshuffle(ids, e2r, D, cap)[0])
    out, cycles, conv = O.reshuffle_refine(ids, e2r, D, cap)
    _valid(ids, e2r, D, cap, out)
    best = O.reshuffle_exact(ids, e2r, D, cap)[1]
    got = O.local_pairs(ids, e2r, out[0])
    assert conv and got == best
    assert greedy <= got and (cycles > 0) == (got > greedy)


def test_refine_cycle_budget():
    r = np.random.default_rng(5)
    T, E, D, k = 120, 32, 8, 4
    p = 1.0 / np.arange(1, E + 1) ** 1.2
    p /= p.sum()
    ids = np.stack([r.choice(E, size=k, replace=False, p=p) for _ in range(T)])
    e2r, _, _ = O.vanilla_placement(E, D)
    cap = T // D
    full, n_full, conv = O.reshuffle_refine(ids, e2r, D, cap)
    assert conv and n_full >= 3
    # no cycle allowed: the greedy, not converged
    zero, n0, c0 = O.reshuffle_refine(ids, e2r, D, cap, 0)
    assert n0 == 0 and not c0
    for a, b in zip(zero, O.reshuffle(ids, e2r, D, cap)):
        assert (a == b).all()
    # every cycle adds local pairs; the budget is respected; exactly n_full cycles converge
    last = O.local_pairs(ids, e2r, zero[0])
    for n in range(1, n_full + 1):
        out, done, c = O.reshuffle_refine(ids, e2r, D, cap, n)
        now = O.local_pairs(ids, e2r, out[0])
        assert done == n and now > last
        _valid(ids, e2r, D, cap, out)
        last = now
    assert c and (out[0] == full[0]).all()
    out, done, c = O.reshuffle_refine(ids, e2r, D, cap, n_full - 1)
    assert not c and done == n_full - 1


def test_refine_without_binding_capacity_changes_nothing():
    ids = WL.uniform_random_ids(150, 16, 2, seed=3)
    e2r, _, _ = O.vanilla_placement(16, 4)
    out, cycles, conv = O.reshuffle_refine(ids, e2r, 4, 150)
    assert cycles == 0 and conv
    for a, b in zip(out, O.reshuffle(ids, e2r, 4, 150)):
        assert (a == b).all()
