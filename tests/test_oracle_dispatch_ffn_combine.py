"""Pins for the oracle's dispatch, expert_ffn, combine and the whole-layer definition."""
import math
import os

import numpy as np
import pytest

from oracle import semmoe_oracle as O
import workloads as WL

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=", 1)
            out[k.strip()] = v.strip()
    return out


def _setup(T=120, E=16, D=4, k=3, seed=0, cap=None, placed=True):
    ids = WL.uniform_random_ids(T, E, k, seed=seed)
    load, co = O.coact_hist(ids, E)
    e2r, phys, inv = O.place(load, co, D) if placed else O.vanilla_placement(E, D)
    cap = cap or -(-T // D)
    tr, shf, ishf, rc = O.reshuffle(ids, e2r, D, cap)
    return ids, e2r, phys, inv, tr, shf, ishf, rc


# ------------------------------------------------------------------ dispatch
@pytest.mark.parametrize("T,E,D,k", [(120, 16, 4, 3), (77, 8, 2, 2), (64, 32, 8, 4)])
def test_dispatch_every_pair_exactly_once_and_counts(T, E, D, k):
    ids, e2r, phys, inv, tr, shf, ishf, rc = _setup(T, E, D, k, seed=T)
    X = np.random.default_rng(0).standard_normal((T, 5)).astype(np.float32)
    o = O.dispatch(X, ids, tr, ishf, phys, D)
    P, m = T * k, E // D
    assert sorted(o["slot_of_pair"]) == list(range(P))                    # each pair dispatched exactly once
    assert (o["pair_of_slot"][o["slot_of_pair"]] == np.arange(P)).all()
    off = o["expert_offsets"]
    assert off[0] == 0 and off[-1] == P and (np.diff(off) >= 0).all()
    load, _ = O.coact_hist(ids, E)
    assert (np.diff(off) == load[inv]).all()                              # physical expert q holds load[expert_of_phys[q]]
    assert (o["rank_offsets"] == off[::m]).all()
    S = o["send_matrix"].astype(np.int64)
    assert S.sum() == P                                                   # per-rank counts sum to T*k
    assert (S.sum(axis=1) == k * rc).all()
    assert (S.sum(axis=0) == np.diff(o["rank_offsets"])).all()
    assert int(o["remote_pairs"]) == P - O.local_pairs(ids, e2r, tr)
    # rows are bit copies
    assert (o["X_perm"] == X[o["pair_of_slot"] // k]).all()
    # each slot's expert is the block it sits in
    q_of_slot = phys[ids.reshape(-1)[o["pair_of_slot"]]]
    for q in range(E):
        assert (q_of_slot[off[q]:off[q + 1]] == q).all()


def test_dispatch_equals_library_stable_argsort_on_composite_key():
    ids, e2r, phys, inv, tr, shf, ishf, rc = _setup(150, 16, 4, 2, seed=9)
    k = 2
    o = O.dispatch(None, ids, tr, ishf, phys, 4)
    P = ids.size
    # visit pairs in shuffled order, then a stable sort by expert
    shuffled_pairs = (shf[:, None].astype(np.int64) * k + np.arange(k)[None, :]).reshape(P)
    q = phys[ids.reshape(P)[shuffled_pairs]]
    want = shuffled_pairs[np.argsort(q, kind="stable")]
    assert (o["pair_of_slot"] == want).all()


def test_dispatch_arrival_order_inside_expert_block():
    """inside an expert block rows come by (source rank, position in that rank's shard)"""
    ids, e2r, phys, inv, tr, shf, ishf, rc = _setup(200, 16, 4, 2, seed=4)
    o = O.dispatch(None, ids, tr, ishf, phys, 4)
    off = o["expert_offsets"]
    for q in range(16):
        toks = o["pair_of_slot"][off[q]:off[q + 1]] // 2
        assert (np.diff(tr[toks]) >= 0).all()
        assert (np.diff(ishf[toks]) > 0).all()


def test_dispatch_hand_example():
    # T=3,k=2,E=4,D=2 (m=2).  placement: experts (1,3) on rank 0, (0,2) on rank 1
    phys = np.array([2, 0, 3, 1])          # phys_of_expert
    ids = np.array([[0, 1], [1, 2], [3, 0]])
    tr = np.array([1, 0, 0])
    ishf = np.array([2, 0, 1])             # shuffled order: token 1, token 2, token 0
    o = O.dispatch(None, ids, tr, ishf, phys, 2)
    # keys q per pair: t0:(2,0) t1:(0,3) t2:(1,2);  p' per pair: t0:(4,5) t1:(0,1) t2:(2,3)
    # sort by (q,p'): q0:{t1j0 p'0, t0j1 p'5} q1:{t2j0} q2:{t2j1 p'3, t0j0 p'4} q3:{t1j1}
    assert list(o["pair_of_slot"]) == [2, 1, 4, 5, 0, 3]
    assert list(o["slot_of_pair"]) == [4, 1, 0, 5, 2, 3]
    assert list(o["expert_offsets"]) == [0, 2, 3, 5, 6] and list(o["rank_offsets"]) == [0, 3, 6]
    assert o["send_matrix"].tolist() == [[2, 2], [1, 1]]
    assert int(o["remote_pairs"]) == 3


def test_uniform_routing_local_rate_is_one_over_D():
    """class-free routing under a balanced placement: LAR = 1/D, the ~25 % baseline the paper's
    Tables 3-4 print for 4 ranks; remote volume follows alpha*k*B*S/G (Sec. 3.1)"""
    g = _golden()
    T, E, D, k = 20000, 16, 4, 2
    ids = WL.uniform_random_ids(T, E, k, seed=77)
    e2r, phys, inv = O.vanilla_placement(E, D)
    tr, shf, ishf, rc = O.home_assignment(T, D)
    o = O.dispatch(None, ids, tr, ishf, phys, D)
    alpha = int(o["remote_pairs"]) / (T * k)
    lar = 1 - alpha
    sigma = math.sqrt(0.25 * 0.75 / (T * k))
    assert abs(lar - 0.25) < 4 * sigma
    assert float(g["baseline_lar_ep4_min"]) - 4 * sigma < lar < float(g["baseline_lar_ep4_max"]) + 4 * sigma
    assert abs(O.remote_fraction(ids, e2r, tr) - alpha) < 1e-15
    # per-device volume alpha*k*T/D == mean over source ranks of remote pairs sent
    S = o["send_matrix"].astype(np.int64)
    assert abs((S.sum() - np.trace(S)) / D - alpha * k * T / D) < 1e-9


def test_load_imbalance_definition():
    S = np.array([[5, 1, 0], [0, 2, 2], [1, 1, 0]])
    assert O.load_imbalance(S) == 6 / 4


# ------------------------------------------------------------------ expert_ffn
def test_swiglu_against_scalar_loops():
    r = np.random.default_rng(1)
    d, F = 5, 4
    x = r.standard_normal((3, d))
    wgu = r.standard_normal((2 * F, d))
    wdn = r.standard_normal((d, F))
    y = O.swiglu_ffn(x, wgu, wdn)
    for n in range(3):
        h = []
        for f in range(F):
            gte = sum(wgu[f, c] * x[n, c] for c in range(d))
            up = sum(wgu[F + f, c] * x[n, c] for c in range(d))
            h.append(gte / (1 + math.exp(-gte)) * up)
        for c in range(d):
            assert abs(y[n, c] - sum(wdn[c, f] * h[f] for f in range(F))) < 1e-12


def test_swiglu_is_linear_in_w_down_and_zero_gate_gives_zero():
    r = np.random.default_rng(2)
    x = r.standard_normal((4, 6))
    wgu = r.standard_normal((8, 6))
    wdn = r.standard_normal((6, 4))
    np.testing.assert_allclose(O.swiglu_ffn(x, wgu, 3 * wdn), 3 * O.swiglu_ffn(x, wgu, wdn), rtol=1e-12)
    wz = wgu.copy()
    wz[:4] = 0
    assert np.abs(O.swiglu_ffn(x, wz, wdn)).max() == 0          # silu(0) = 0


def test_expert_ffn_blocks_use_the_original_experts_weights_and_leave_other_ranks():
    ids, e2r, phys, inv, tr, shf, ishf, rc = _setup(90, 8, 4, 2, seed=5)
    d, F = 6, 5
    r = np.random.default_rng(3)
    X = r.standard_normal((90, d))
    W = {e: (r.standard_normal((2 * F, d)), r.standard_normal((d, F))) for e in range(8)}
    o = O.dispatch(X, ids, tr, ishf, phys, 4)
    Y = np.full((180, d), 777.0)
    O.expert_ffn(o["X_perm"], o["expert_offsets"], inv, lambda e: W[e], 4, rank=1, Y=Y)
    lo, hi = o["rank_offsets"][1], o["rank_offsets"][2]
    assert (Y[:lo] == 777.0).all() and (Y[hi:] == 777.0).all()
    for s in range(lo, hi):
        p = o["pair_of_slot"][s]
        e = ids.reshape(-1)[p]
        np.testing.assert_allclose(Y[s], O.swiglu_ffn(X[p // 2][None], *W[e])[0], rtol=1e-10, atol=1e-13)


# ------------------------------------------------------------------ combine
@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_combine_after_dispatch_is_identity_for_unit_weights(k):
    T, E, D = 70, 16, 4
    ids, e2r, phys, inv, tr, shf, ishf, rc = _setup(T, E, D, k, seed=k)
    X = WL.round_to_bf16(np.random.default_rng(k).standard_normal((T, 9)).astype(np.float32))
    o = O.dispatch(X, ids, tr, ishf, phys, D)
    out = O.combine(o["X_perm"], o["slot_of_pair"], np.ones((T, k)))
    assert (out == k * X.astype(np.float64)).all()
    onehot = np.zeros((T, k))
    onehot[:, k - 1] = 1
    assert (O.combine(o["X_perm"], o["slot_of_pair"], onehot) == X).all()


def test_combine_weights_and_shared_term():
    Y = np.arange(12, dtype=np.float64).reshape(6, 2)
    slot = np.array([5, 0, 2, 3, 1, 4])
    w = np.array([[0.5, 2.0], [1.0, -1.0], [0.0, 3.0]])
    sh = np.ones((3, 2))
    out = O.combine(Y, slot, w, sh)
    assert out.tolist() == [[0.5 * 10 + 2 * 0 + 1, 0.5 * 11 + 2 * 1 + 1],
                            [4 - 6 + 1, 5 - 7 + 1],
                            [3 * 8 + 1, 3 * 9 + 1]]


# ------------------------------------------------------------------ whole layer == plain definition
@pytest.mark.parametrize("placed,shuffle,cf", [(False, False, 1.0), (True, False, 1.0), (True, True, 1.0),
                                               (True, True, 2.0)])
def test_path_equals_plain_moe_definition(placed, shuffle, cf):
    """lossless (Sec. 5): placement, reshuffle and capacity never change the layer output"""
    w = WL.small(T=60, d=16, E=8, k=2, F=12, D=4, dtype="fp32")
    X = WL.hidden(w)
    L = O.route_logits(X, WL.router_weight(w), None, WL.token_class(w), WL.class_bias(w))
    ids, tw = O.select_topk(L, w.k, "softmax", True)
    weights = {e: WL.expert_weight(w, e) for e in range(w.E)}
    shared = WL.shared_weight(w)
    load, co = O.coact_hist(ids, w.E)
    e2r, phys, inv = O.place(load, co, w.D) if placed else O.vanilla_placement(w.E, w.D)
    cap = int(math.ceil(cf * w.T / w.D))
    tr, shf, ishf, rc = O.reshuffle(ids, e2r, w.D, cap) if shuffle else O.home_assignment(w.T, w.D)
    o = O.dispatch(X, ids, tr, ishf, phys, w.D)
    Y = O.expert_ffn(o["X_perm"], o["expert_offsets"], inv, lambda e: weights[e], w.D)
    out = O.combine(Y, o["slot_of_pair"], tw, O.swiglu_ffn(X, *shared))
    ref = O.moe_definition(X, ids, tw, lambda e: weights[e], shared)
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("with_shared,sample", [(True, None), (False, [3, 17, 17, 40, 0]), (True, [59])])
def test_expert_major_definition_equals_token_major_definition(with_shared, sample):
    """`moe_definition_by_expert` is the same sum in another order; every expert's weights are asked for once,
    in ascending id, and only those of experts a sampled token uses"""
    w = WL.small(T=60, d=16, E=8, k=3, F=12, D=4, dtype="fp32")
    X = WL.hidden(w)
    L = O.route_logits(X, WL.router_weight(w), None, WL.token_class(w), WL.class_bias(w))
    ids, tw = O.select_topk(L, w.k, "softmax", False)
    weights = {e: WL.expert_weight(w, e) for e in range(w.E)}
    shared = WL.shared_weight(w) if with_shared else None
    asked = []

    def weight_of(e):
        asked.append(e)
        return weights[e]

    got = O.moe_definition_by_expert(X, ids, tw, weight_of, shared, tokens=sample)
    ref = O.moe_definition(X, ids, tw, lambda e: weights[e], shared, tokens=sample)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-15)
    used = sorted(set(ids.ravel().tolist())) if sample is None else sorted(set(ids[sample].ravel().tolist()))
    assert asked == used
    # a dropped weight, a wrong expert or a doubled term cannot hide: one token, by hand
    i = 7
    by_hand = sum(tw[i, j] * O.swiglu_ffn(X[i:i + 1], *weights[int(ids[i, j])])[0] for j in range(w.k))
    if shared is not None:
        by_hand = by_hand + O.swiglu_ffn(X[i:i + 1], *shared)[0]
    np.testing.assert_allclose(O.moe_definition_by_expert(X, ids, tw, lambda e: weights[e], shared, tokens=[i])[0],
                               by_hand, rtol=1e-12, atol=1e-15)


def test_semantic_placement_and_reshuffle_raise_local_rate_on_config1():
    """the method's point (Sec. 4.5): co-scheduling raises the local activation rate over vanilla"""
    w = WL.CONFIGS["c1_tiny_fp32"]
    Wr, cb = WL.router_weight(w), WL.class_bias(w)
    Lp = O.route_logits(WL.hidden(w, profile=True), Wr, None, WL.token_class(w, profile=True), cb)
    idp, _ = O.select_topk(Lp, w.k, w.score, w.renorm)
    e2r, phys, inv = O.place(*O.coact_hist(idp, w.E), w.D)
    L = O.route_logits(WL.hidden(w), Wr, None, WL.token_class(w), cb)
    ids, _ = O.select_topk(L, w.k, w.score, w.renorm)
    home = O.home_rank(w.T, w.D)
    v_e2r, _, _ = O.vanilla_placement(w.E, w.D)
    lar_vanilla = 1 - O.remote_fraction(ids, v_e2r, home)
    lar_placed = 1 - O.remote_fraction(ids, e2r, home)
    tr, *_ = O.reshuffle(ids, e2r, w.D, w.cap)
    lar_full = 1 - O.remote_fraction(ids, e2r, tr)
    assert abs(lar_vanilla - 0.25) < 0.08 and abs(lar_placed - 0.25) < 0.08   # home ranks know nothing
    assert lar_full > 0.85
    _, val = O.reshuffle_exact(ids, e2r, w.D, w.cap)
    assert O.local_pairs(ids, e2r, tr) <= val


# ------------------------------------------------------------------ inputs
def test_workload_generators_are_seeded_and_shaped():
    w = WL.CONFIGS["c1_tiny_fp32"]
    assert (WL.hidden(w) == WL.hidden(w)).all() and WL.hidden(w).shape == (256, 512)
    assert not (WL.hidden(w)[:8] == WL.hidden(w, profile=True)[:8]).all()
    cl = WL.class_clusters(w)
    assert sorted(cl.reshape(-1)) == list(range(16))            # disjoint clusters on config 1
    cb = WL.class_bias(w)
    assert ((cb == 2.0).sum(axis=1) == 4).all() and ((cb == 0) | (cb == 2.0)).all()
    w4 = WL.CONFIGS["c4_gpt_oss_120b"]
    tc = WL.token_class(w4)
    assert abs((tc < 0).mean() - 0.10) < 0.01 and tc.max() == 31
    w2 = WL.CONFIGS["c2_qwen3_30b"]
    x = WL.hidden(w2, n=64)
    assert (WL.round_to_bf16(x) == x).all()                      # already bf16-representable
    b = WL.f32_to_bf16_bits(x)
    assert (WL.bf16_bits_to_f32(b) == x).all()


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, 1.005859375], dtype=np.float32)   # 1, 1+2^-8 (tie), 1+3*2^-8 (tie), 1+1.5*2^-8
    r = WL.round_to_bf16(x)
    assert list(r) == [1.0, 1.0, 1.015625, 1.0078125]
