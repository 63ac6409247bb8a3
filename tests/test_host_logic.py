"""CPU-only tests of the library's host side: it loads, exports every declared symbol, validates
arguments before touching a GPU, sizes its workspace, and its host placement solver equals the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2503_04398_amd as S
from paper_2503_04398_amd import binding as B
from oracle import semmoe_oracle as O
import workloads as WL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "semmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(semmoe_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = S.load_library()
    declared = _declared_symbols()
    assert len(declared) >= 12
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTS) == declared          # the binding covers exactly the header
    assert lib.semmoe_version() >= 100


def _mk(**kw):
    base = dict(T=64, d=64, E=16, k=2, F=32, D=4, cap=16)
    base.update(kw)
    return S.SemMoE(S.Config(**base), allocate_workspace=False)


def test_tuning_knobs_are_process_state_that_reads_back():
    """a knob holds its value until it is set again (from any SemMoE object: the state belongs to the process),
    reads back, and is restored by a negative value; keys outside the table are refused"""
    a, b = _mk(), _mk(T=128, cap=32)
    for key in range(8):
        assert a.get_tuning(key) == -1
    try:
        a.set_tuning(4, 13)
        assert a.get_tuning(4) == 13 and b.get_tuning(4) == 13
        b.set_tuning(4, 7)
        assert a.get_tuning(4) == 7
    finally:
        a.set_tuning(4, -1)
    assert b.get_tuning(4) == -1
    assert a.lib.semmoe_set_tuning(8, 1) == -1 and a.lib.semmoe_set_tuning(-1, 1) == -1
    v = C.c_int32(5)
    assert a.lib.semmoe_get_tuning(8, C.byref(v)) == -1 and a.lib.semmoe_get_tuning(0, None) == -1


def test_workspace_bytes_grows_with_the_hidden_activation():
    a = _mk().workspace_bytes()
    b = _mk(T=128, cap=32).workspace_bytes()
    assert b > a >= 64 * 2 * 32 * 2


@pytest.mark.parametrize("kw,status", [
    (dict(E=15), -2),                 # E % D
    (dict(k=17, E=32), -5),           # k above the kernel limit
    (dict(k=16, E=8, D=4), -2),       # k > E
    (dict(d=60), -2),                 # d % 8
    (dict(F=12), -2),                 # F % 8
    (dict(dtype=7), -5),
    (dict(score=3), -5),
    (dict(E=1024, D=4), -5),
    (dict(D=0), -1),
])
def test_workspace_bytes_rejects_bad_shapes(kw, status):
    with pytest.raises(S.SemMoEError) as ei:
        _mk(**kw).workspace_bytes()
    assert ei.value.status == status


def test_calls_reject_null_pointers_and_bad_capacity_without_a_gpu():
    m = _mk()
    lib = m.lib
    c = m.cfg.c()
    one = np.zeros(4096, dtype=np.int32)
    p = one.ctypes.data
    assert lib.semmoe_route_from_logits(C.byref(c), None, None, None, p, p) == -1
    assert lib.semmoe_coact_hist(C.byref(c), None, None, 4, p, p) == -1
    assert lib.semmoe_coact_hist(C.byref(c), None, p, -1, p, p) == -1
    assert lib.semmoe_combine(C.byref(c), None, None, p, p, None, p) == -1
    assert lib.semmoe_reshuffle(C.byref(c), None, p, p, p, p, p, None, p, 1 << 20) == -1
    c.cap = 15                                   # cap * D < T
    assert lib.semmoe_reshuffle(C.byref(c), None, p, p, p, p, p, p, p, 1 << 20) == -2
    c.cap = 16
    assert lib.semmoe_reshuffle(C.byref(c), None, p, p, p, p, p, p, None, 0) == -3      # no workspace
    assert lib.semmoe_reshuffle(C.byref(c), None, p, p, p, p, p, p, p, 8) == -3         # too small
    # the allocation-free form checks the same things, and its size limit, before it touches a GPU
    assert lib.semmoe_reshuffle_static(C.byref(c), None, p, p, p, p, p, None) == -1
    c.cap = 15
    assert lib.semmoe_reshuffle_static(C.byref(c), None, p, p, p, p, p, p) == -2
    c.cap = 16
    big = S.Config(T=1 << 21, d=64, E=64, k=8, F=32, D=32, cap=1 << 16).c()      # scratch need above the fixed array
    assert S.SemMoE(S.Config(T=1 << 21, d=64, E=64, k=8, F=32, D=32, cap=1 << 16),
                    allocate_workspace=False).workspace_bytes() > (4 << 20)
    assert lib.semmoe_reshuffle_static(C.byref(big), None, p, p, p, p, p, p) == -5
    assert lib.semmoe_expert_ffn(C.byref(c), None, 4, p, p, p, p, p, p, p, 1 << 20) == -1   # rank >= D
    assert lib.semmoe_expert_ffn(C.byref(c), None, 0, p + 4, p, p, p, p, p, p, 1 << 20) == -1  # misaligned rows
    assert lib.semmoe_route(C.byref(c), None, p, p, None, p, None, None, None, p, p, p, 1 << 20) == -1  # class pair
    c.score, c.n_group, c.topk_group = 1, 3, 1   # E % n_group
    assert lib.semmoe_route_from_logits(C.byref(c), None, p, None, p, p) == -2
    c.n_group, c.topk_group, c.k = 8, 1, 4        # k > topk_group * E / n_group
    assert lib.semmoe_route_from_logits(C.byref(c), None, p, None, p, p) == -2
    assert lib.semmoe_workspace_bytes(None, None) == -1


def test_next_row_calls_reject_bad_arguments_without_a_gpu():
    """the entry points of the widened rows validate before they launch anything"""
    m = _mk()
    lib = m.lib
    c = m.cfg.c()
    one = np.zeros(4096, dtype=np.int32)
    p = one.ctypes.data
    big = 1 << 20
    # reshuffle with spill rounds
    assert lib.semmoe_reshuffle_rounds(C.byref(c), None, p, p, 0, p, p, p, p, p, big) == -1          # rounds < 1
    assert lib.semmoe_reshuffle_rounds(C.byref(c), None, None, p, 2, p, p, p, p, p, big) == -1
    assert lib.semmoe_reshuffle_rounds(C.byref(c), None, p, p, 2, p, p, p, p, None, 0) == -3
    # reshuffle refined to the optimum
    assert lib.semmoe_reshuffle_refine(C.byref(c), None, p, p, 1, 10, p, p, p, p, None, p, big) == -1   # no info
    assert lib.semmoe_reshuffle_refine(C.byref(c), None, p, p, 1, -1, p, p, p, p, p, p, big) == -1      # max_cycles < 0
    assert lib.semmoe_reshuffle_refine(C.byref(c), None, p, p, 0, 10, p, p, p, p, p, p, big) == -1      # rounds < 1
    assert lib.semmoe_reshuffle_refine(C.byref(c), None, p, None, 1, 10, p, p, p, p, p, p, big) == -1
    assert lib.semmoe_reshuffle_refine(C.byref(c), None, p, p, 1, 10, p, p, p, p, p, None, 0) == -3
    assert lib.semmoe_reshuffle_refine(None, None, p, p, 1, 10, p, p, p, p, p, p, big) == -1
    keep = (c.T, c.D, c.cap)
    c.T, c.cap = 32769, 32769
    assert lib.semmoe_reshuffle_refine(C.byref(c), None, p, p, 1, 10, p, p, p, p, p, p, big) == -5      # T > 32768
    c.T, c.D, c.cap = keep
    c.D, c.E, c.cap = 32, 32, 2
    assert lib.semmoe_reshuffle_refine(C.byref(c), None, p, p, 1, 10, p, p, p, p, p, p, big) == -5      # D > 16
    c.D, c.E, c.cap = keep[1], 16, keep[2]
    # activation table, schedule tables, table-driven reshuffle
    assert lib.semmoe_token_expert_hist(C.byref(c), None, None, p, 4, 8, p) == -1
    assert lib.semmoe_token_expert_hist(C.byref(c), None, p, p, -1, 8, p) == -1
    assert lib.semmoe_token_expert_hist(C.byref(c), None, p, p, 4, 0, p) == -1                       # empty vocabulary
    assert lib.semmoe_lookup_tables(C.byref(c), None, p, 8, p, p, p) == -1
    assert lib.semmoe_lookup_tables(C.byref(c), p, p, 0, p, p, p) == -1
    assert lib.semmoe_reshuffle_lookup(C.byref(c), None, p, 0, p, p, p, 0, p, p, p, p, p, big) == -1  # V <= 0
    assert lib.semmoe_reshuffle_lookup(C.byref(c), None, p, 8, None, p, p, 0, p, p, p, p, p, big) == -1
    assert lib.semmoe_reshuffle_lookup(C.byref(c), None, p, 8, p, p, p, 0, p, p, p, p, p, 8) == -3
    c.cap = 15
    assert lib.semmoe_reshuffle_lookup(C.byref(c), None, p, 8, p, p, p, 0, p, p, p, p, p, big) == -2  # cap * D < T
    c.cap = 16
    # both tables
    assert lib.semmoe_reshuffle_cond(C.byref(c), None, p, 8, p, p, p, p, 0, p, p, p, 0, p, p, p, p, p, big) == -1  # VA <= 0
    assert lib.semmoe_reshuffle_cond(C.byref(c), None, p, 8, p, p, p, None, 8, p, p, p, 0, p, p, p, p, p, big) == -1
    assert lib.semmoe_reshuffle_cond(C.byref(c), None, p, 8, p, p, p, p, 8, p, p, p, 0, p, p, p, p, p, 8) == -3
    assert lib.semmoe_device_sequence(C.byref(c), None, None, p, 4, None, p) == -1
    assert lib.semmoe_device_sequence(C.byref(c), None, p, p, -1, None, p) == -1
    assert lib.semmoe_device_sequence(C.byref(c), None, p, p, 4, None, None) == -1
    assert lib.semmoe_device_sequence(C.byref(c), None, p, p, 0, None, p) == 0                       # nothing to do
    # request scheduling
    assert lib.semmoe_request_schedule(C.byref(c), None, None, 3, p, 8, p, p, p, p, p, p, p, big) == -1
    assert lib.semmoe_request_schedule(C.byref(c), None, p, -1, p, 8, p, p, p, p, p, p, p, big) == -1
    assert lib.semmoe_request_schedule(C.byref(c), None, p, 3, p, 0, p, p, p, p, p, p, p, big) == -1
    assert lib.semmoe_request_schedule(C.byref(c), None, p, 65, p, 8, p, p, p, p, p, p, p, big) == -2  # n_req > T
    assert lib.semmoe_request_schedule(C.byref(c), None, p, 0, p, 8, p, p, p, p, p, p, p, big) == -2   # tokens, no request
    assert lib.semmoe_request_schedule(C.byref(c), None, p, 3, p, 8, p, p, p, p, p, p, None, 0) == -3
    assert lib.semmoe_set_tuning(99, 1) == -1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_LIB", None)
    monkeypatch.setenv("SEMMOE_LIB", str(tmp_path / "nope.so"))
    with pytest.raises(S.SemMoEError):
        B.load_library()
    monkeypatch.delenv("SEMMOE_LIB")
    monkeypatch.setattr(B, "_LIB", None)
    assert B.load_library() is not None


# ------------------------------------------------------------------ host placement solver == oracle
def _clustered_ids(T, E, D, k, seed, noise):
    r = np.random.default_rng(seed)
    m = E // D
    pi = r.permutation(E)
    ids = np.zeros((T, k), dtype=np.int32)
    for i in range(T):
        if r.random() < noise:
            ids[i] = r.choice(E, k, replace=False)
        else:
            c = r.integers(0, D)
            ids[i] = pi[c * m + r.choice(m, min(k, m), replace=False)] if k <= m else r.choice(E, k, replace=False)
    return ids


@pytest.mark.parametrize("E,D,k,noise,alpha,gamma,ft", [
    (16, 4, 2, 0.2, 1, 0, 8), (32, 8, 4, 0.5, 1, 0, 8), (24, 3, 3, 0.7, 1, 0, 0), (32, 4, 4, 0.6, 2, 1, 3),
    (64, 8, 8, 0.4, 1, 0, 8), (16, 1, 2, 0.5, 1, 0, 8), (16, 16, 2, 0.5, 1, 0, 8),
    (32, 4, 4, 0.6, 1, 2, 8), (48, 8, 4, 0.5, 4, 1, 8), (24, 3, 3, 0.7, 0, 1, 8), (64, 8, 8, 0.4, 16, 1, 4),
])
def test_host_place_equals_oracle(E, D, k, noise, alpha, gamma, ft):
    ids = _clustered_ids(700, E, D, k, seed=E * 7 + D, noise=noise)
    load, co = O.coact_hist(ids, E)
    want = O.place(load, co, D, alpha, gamma, ft)
    m = S.SemMoE(S.Config(T=1, d=8, E=E, k=k, F=8, D=D, cap=1), allocate_workspace=False)
    got = m.place(load, co, alpha, gamma, ft)
    for g, w_ in zip(got, want):
        assert (g == w_).all()


def test_host_place_equals_oracle_on_config2_profile_routing():
    w = WL.CONFIGS["c2_qwen3_30b"]
    n = 2048
    L = O.route_logits(WL.hidden(w, True, n), WL.router_weight(w), None, WL.token_class(w, True, n), WL.class_bias(w))
    # vectorised top-k stands in for the oracle's row loop here; ties are absent in continuous logits
    ids = np.argsort(-L, axis=1, kind="stable")[:, :w.k].astype(np.int32)
    load, co = O.coact_hist(ids, w.E)
    want = O.place(load, co, w.D)
    got = S.SemMoE(S.Config.from_workload(w), allocate_workspace=False).place(load, co)
    for g, w_ in zip(got, want):
        assert (g == w_).all()


@pytest.mark.parametrize("V,E,D,k,seed", [(40, 16, 4, 2, 0), (300, 64, 8, 8, 1), (17, 8, 1, 2, 2), (64, 32, 32, 4, 3),
                                          (128, 48, 3, 16, 4)])
def test_host_lookup_tables_equal_oracle(V, E, D, k, seed):
    """schedule table, confidence and keep priority from an activation table: integer for integer; the table has
    unseen keys, ties between ranks and single-activation keys"""
    r = np.random.default_rng(seed)
    table = r.integers(0, 6, size=(V, E)).astype(np.int64) * (r.random((V, E)) < 0.3)
    table[0] = 0                      # never profiled
    table[1] = 0
    table[1, :2] = 1                  # two experts once each: a tie between ranks when they sit apart
    if V > 2:
        table[2] = 0
        table[2, E - 1] = 1           # a single activation
    e2r = (r.permutation(E) % D).astype(np.int32)
    want = O.lookup_tables(table, e2r, D, k)
    m = S.SemMoE(S.Config(T=1, d=8, E=E, k=k, F=8, D=D, cap=1), allocate_workspace=False)
    got = m.lookup_tables(table.astype(np.uint32), e2r)
    for g, w_, name in zip(got, want, ("dev", "conf_q16", "level")):
        assert g.dtype == np.int32 and (g == w_).all(), name
    assert got[0][0] == -1 and got[1][0] == 0 and got[2][0] == 0


def test_host_lookup_tables_reject_bad_arguments():
    m = S.SemMoE(S.Config(T=1, d=8, E=8, k=2, F=8, D=4, cap=1), allocate_workspace=False)
    with pytest.raises(S.SemMoEError) as ei:
        m.lookup_tables(np.ones((4, 8), dtype=np.uint32), np.full(8, 4, dtype=np.int32))   # rank out of range
    assert ei.value.status == -1


def test_host_place_rejects_bad_arguments():
    m = S.SemMoE(S.Config(T=1, d=8, E=15, k=2, F=8, D=4, cap=1), allocate_workspace=False)
    with pytest.raises(S.SemMoEError) as ei:
        m.place(np.ones(15), np.eye(15))
    assert ei.value.status == -2


# ------------------------------------------------------------------ host co-scheduling solver == oracle
def _units(T, E, D, k, U, seed, noise):
    """units = runs of tokens (requests) of one topic over clustered routing; returns load, coact, unit_act, unit_len"""
    r = np.random.default_rng(seed)
    ids = _clustered_ids(T, E, D, k, seed, noise)
    cuts = np.sort(r.choice(np.arange(1, T), size=U - 1, replace=False))
    off = np.concatenate([[0], cuts, [T]])
    unit_of = np.repeat(np.arange(U), np.diff(off))
    load, co = O.coact_hist(ids, E)
    return load, co, O.token_expert_table(unit_of, ids, U, E), np.diff(off), off


@pytest.mark.parametrize("E,D,k,U,noise,prm", [
    (16, 4, 2, 10, 0.3, dict(alpha_e=1, beta_e=1, gamma_e=0, alpha_r=0, beta_r=1, ft_passes=4, n_steps=3, w_load=1, w_comm=1)),
    (32, 8, 4, 37, 0.5, dict(alpha_e=2, beta_e=3, gamma_e=1, alpha_r=1, beta_r=50, ft_passes=2, n_steps=4, w_load=2, w_comm=1)),
    (24, 3, 3, 7, 0.7, dict(alpha_e=1, beta_e=0, gamma_e=0, alpha_r=1, beta_r=0, ft_passes=0, n_steps=1, w_load=0, w_comm=1)),
    (16, 1, 2, 5, 0.5, dict(alpha_e=1, beta_e=1, gamma_e=0, alpha_r=0, beta_r=1, ft_passes=8, n_steps=2, w_load=1, w_comm=1)),
    (16, 16, 2, 3, 0.5, dict(alpha_e=1, beta_e=2, gamma_e=0, alpha_r=1, beta_r=1, ft_passes=8, n_steps=2, w_load=1, w_comm=0)),
    (64, 8, 8, 24, 0.4, dict(alpha_e=0, beta_e=1, gamma_e=0, alpha_r=0, beta_r=1, ft_passes=1, n_steps=2, w_load=1, w_comm=4)),
])
def test_host_coschedule_equals_oracle(E, D, k, U, noise, prm):
    load, co, act, ln, _ = _units(500, E, D, k, U, seed=E + 3 * D + U, noise=noise)
    want_e2r, want_ur, want_scores, want_best = O.coschedule(load, co, act, ln, D, **prm)
    m = S.SemMoE(S.Config(T=1, d=8, E=E, k=k, F=8, D=D, cap=1), allocate_workspace=False)
    e2r, phys, inv, ur, scores, best = m.coschedule(load, co, act, ln, **prm)
    assert e2r.tolist() == want_e2r.tolist()
    assert ur.tolist() == want_ur.tolist()
    assert scores.tolist() == want_scores and best == want_best
    want_phys, want_inv = O.placement_order(want_e2r, D)
    assert phys.tolist() == want_phys.tolist() and inv.tolist() == want_inv.tolist()


def test_host_coschedule_with_no_request_weight_and_one_step_places_like_place():
    """beta_e = 0: the placement of every step is `place`'s, whatever the units are"""
    load, co, act, ln, _ = _units(400, 32, 4, 4, 9, seed=5, noise=0.4)
    m = S.SemMoE(S.Config(T=1, d=8, E=32, k=4, F=8, D=4, cap=1), allocate_workspace=False)
    e2r, phys, inv, _, _, _ = m.coschedule(load, co, act, ln, alpha_e=1, beta_e=0, gamma_e=0, n_steps=2)
    want = m.place(load, co, 1, 0, 8)
    assert e2r.tolist() == want[0].tolist() and phys.tolist() == want[1].tolist() and inv.tolist() == want[2].tolist()


def test_host_coschedule_rejects_bad_arguments():
    m = S.SemMoE(S.Config(T=1, d=8, E=8, k=2, F=8, D=4, cap=1), allocate_workspace=False)
    load, co = np.ones(8), np.ones((8, 8))
    act, ln = np.ones((3, 8)), np.ones(3)
    for bad, status in [(dict(n_steps=0), -1), (dict(ft_passes=-1), -1), (dict(w_load=-1), -1),
                        (dict(beta_e=1 << 21), -5)]:
        with pytest.raises(S.SemMoEError) as ei:
            m.coschedule(load, co, act, ln, **bad)
        assert ei.value.status == status, bad
    with pytest.raises(S.SemMoEError) as ei:
        m.coschedule(load, co, np.full((3, 8), 1 << 38, dtype=np.uint64), ln)          # total mass >= 2^40
    assert ei.value.status == -5
    m15 = S.SemMoE(S.Config(T=1, d=8, E=15, k=2, F=8, D=4, cap=1), allocate_workspace=False)
    with pytest.raises(S.SemMoEError) as ei:
        m15.coschedule(np.ones(15), np.ones((15, 15)), np.ones((3, 15)), ln)
    assert ei.value.status == -2


@pytest.mark.parametrize("V,D,k,n_req,seed", [(30, 4, 2, 9, 0), (200, 8, 8, 40, 1), (5, 1, 3, 2, 2), (64, 32, 4, 100, 3)])
def test_host_token_labels_equal_oracle(V, D, k, n_req, seed):
    r = np.random.default_rng(seed)
    lens = r.integers(0, 30, size=n_req)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = r.integers(-1, V + 1, size=int(off[-1])).astype(np.int32)          # some keys outside the table
    keys[keys == V - 1] = 0                                                   # the last id never occurs
    rr = r.integers(0, D, size=n_req).astype(np.int32)
    want = O.token_labels(off, keys, rr, V, D, k)
    m = S.SemMoE(S.Config(T=1, d=8, E=max(D, k), k=k, F=8, D=D, cap=1), allocate_workspace=False)
    got = m.token_labels(off, keys, rr, V)
    for g, w_, name in zip(got, want, ("dev", "conf_q16", "level")):
        assert g.dtype == np.int32 and g.tolist() == w_.tolist(), name
    assert got[0][V - 1] == -1


def test_host_token_labels_reject_bad_arguments():
    m = S.SemMoE(S.Config(T=1, d=8, E=8, k=2, F=8, D=4, cap=1), allocate_workspace=False)
    with pytest.raises(S.SemMoEError) as ei:
        m.token_labels(np.array([0, 2, 1]), np.zeros(2), np.array([0, 0]), 4)      # offsets decrease
    assert ei.value.status == -1
    with pytest.raises(S.SemMoEError) as ei:
        m.token_labels(np.array([0, 1, 2]), np.zeros(2), np.array([0, 4]), 4)      # rank out of range
    assert ei.value.status == -1


def test_host_coschedule_equals_oracle_at_config2_shape():
    """128 experts on 8 clusters, 34 requests cut from 8192 tokens of clustered top-8 routing"""
    load, co, act, ln, _ = _units(8192, 128, 8, 8, 34, seed=11, noise=0.5)
    prm = dict(alpha_e=1, beta_e=1, gamma_e=0, alpha_r=0, beta_r=1, ft_passes=1, n_steps=2, w_load=1, w_comm=1)
    want_e2r, want_ur, want_scores, want_best = O.coschedule(load, co, act, ln, 8, **prm)
    m = S.SemMoE(S.Config(T=1, d=8, E=128, k=8, F=8, D=8, cap=1), allocate_workspace=False)
    e2r, _, _, ur, scores, best = m.coschedule(load, co, act, ln, **prm)
    assert e2r.tolist() == want_e2r.tolist() and ur.tolist() == want_ur.tolist()
    assert scores.tolist() == want_scores and best == want_best


def test_config_accepts_the_names_of_its_enumerations():
    c = S.Config(T=8, d=8, E=8, k=2, F=8, D=2, score="sigmoid", dtype="fp32")
    assert c.score == B.SIGMOID and c.dtype == B.FP32 and c.c().score == B.SIGMOID
    assert S.Config(T=8, d=8, E=8, k=2, F=8, D=2, score="softmax", dtype="bf16").c().dtype == B.BF16
    for bad in (dict(score="tanh"), dict(dtype="fp16")):
        with pytest.raises(ValueError):
            S.Config(T=8, d=8, E=8, k=2, F=8, D=2, **bad)
