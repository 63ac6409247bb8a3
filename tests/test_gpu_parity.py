"""GPU parity: every step of the HIP path against the CPU oracle, through the C ABI.

Integer and index outputs are compared bit for bit; floats with max|a-b|/max|b| <= 1e-5 (fp32) or
2e-2 (bf16).  Sizes here are the ones the oracle finishes in seconds; they span several tiles and
ragged tails.  Full-size configurations are in test_gpu_configs.py.
"""
import math

import numpy as np
import pytest
import torch

import workloads as WL
from oracle import semmoe_oracle as O
import paper_2503_04398_amd as S
from tests import harness as H

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


@pytest.fixture(params=[1, 2, 3], ids=["multi_wg", "single_wg", "two_launch"])
def index_path(request):
    """run the test with each implementation of the index kernels (reshuffle, dispatch index)"""
    m = S.SemMoE(S.Config(T=1, d=8, E=2, k=1, F=8, D=1, cap=1), allocate_workspace=False)
    m.set_tuning(3, request.param)
    yield request.param
    m.set_tuning(3, -1)


# ------------------------------------------------------------------------------------------- route
@pytest.mark.parametrize("E,k,T,renorm", [(16, 2, 100, False), (128, 8, 300, True), (256, 8, 77, True),
                                           (64, 1, 65, True), (200, 5, 33, False), (512, 16, 40, True),
                                           (256, 16, 1000, True), (24, 3, 9, False), (128, 8, 8193, True)])
def test_route_from_logits_softmax(E, k, T, renorm):
    _say("route_from_logits softmax", E, k, T, renorm)
    r = np.random.default_rng(E + k)
    L = (2 * r.standard_normal((T, E))).astype(np.float32)
    L[0, :] = 0.25                       # a full tie row: lowest ids win
    L[1, E // 2:] = L[1, :E - E // 2]    # pairwise ties
    L[2] = np.round(L[2])                # many ties
    cfg = S.Config(T=T, d=8, E=E, k=k, F=8, D=1, renorm=renorm, cap=T)
    m = S.SemMoE(cfg, allocate_workspace=False)
    ids = torch.empty(T, k, dtype=torch.int32, device=H.DEV)
    w = torch.empty(T, k, dtype=torch.float32, device=H.DEV)
    m.route_from_logits(H.to_dev(L), ids, w)
    torch.cuda.synchronize()
    want_ids, want_w = O.select_topk(L, k, "softmax", renorm)
    assert (H.to_np(ids) == want_ids).all()
    assert O.max_rel_err(H.to_np(w), want_w) <= 1e-5


@pytest.mark.parametrize("E,k,T,ng,tg,scale,bias", [(256, 8, 200, 8, 4, 2.5, True), (64, 6, 90, 4, 2, 1.0, False),
                                                     (32, 4, 70, 1, 1, 1.0, True), (128, 8, 50, 16, 3, 1.0, True),
                                                     (16, 2, 40, 16, 4, 1.0, False), (240, 6, 50, 5, 2, 1.0, True),
                                                     (256, 16, 30, 8, 8, 0.5, True), (40, 3, 20, 20, 5, 1.0, False),
                                                     (96, 7, 333, 6, 3, 1.0, True)])
def test_route_from_logits_sigmoid_group_limited(E, k, T, ng, tg, scale, bias):
    _say("route_from_logits sigmoid", E, k, T, ng, tg)
    r = np.random.default_rng(E * 3 + k)
    L = (1.7 * r.standard_normal((T, E))).astype(np.float32)
    L[0, :] = 0.0
    L[1] = np.round(L[1])
    L[2, 0] = 40.0                       # beyond the clamp
    L[2, 1] = -40.0
    sb = (0.05 * r.standard_normal(E)).astype(np.float32) if bias else None
    cfg = S.Config(T=T, d=8, E=E, k=k, F=8, D=1, score=S.binding.SIGMOID, renorm=True, n_group=ng, topk_group=tg,
                   routed_scale=scale, cap=T)
    m = S.SemMoE(cfg, allocate_workspace=False)
    ids = torch.empty(T, k, dtype=torch.int32, device=H.DEV)
    w = torch.empty(T, k, dtype=torch.float32, device=H.DEV)
    m.route_from_logits(H.to_dev(L), ids, w, sel_bias=None if sb is None else H.to_dev(sb))
    torch.cuda.synchronize()
    want_ids, want_w = O.select_topk(L, k, "sigmoid", True, ng, tg, scale, sb)
    got = H.to_np(ids)
    assert (got == want_ids).all(), np.argwhere(got != want_ids)[:5]
    assert O.max_rel_err(H.to_np(w), want_w) <= 1e-5


@pytest.mark.parametrize("dtype,T,d,E,k,split", [
    ("fp32", 200, 72, 16, 2, -1), ("bf16", 333, 200, 128, 8, -1), ("bf16", 333, 200, 128, 8, 0),
    ("bf16", 130, 64, 24, 3, -1), ("fp32", 64, 512, 16, 2, -1), ("bf16", 257, 1032, 256, 8, -1),
    ("bf16", 257, 1032, 256, 8, 0), ("bf16", 100, 4096, 128, 8, 5), ("bf16", 40, 512, 384, 6, 3),
    ("bf16", 700, 256, 64, 4, -1), ("bf16", 512, 2048, 128, 8, 16), ("bf16", 16400, 136, 64, 4, -1),
    ("bf16", 16390, 72, 256, 8, -1), ("bf16", 32800, 72, 128, 8, -1),
    ("bf16", 12300, 2560, 256, 8, -1), ("bf16", 8200, 1024, 256, 8, 102), ("bf16", 700, 1536, 256, 8, 103),
    ("bf16", 300, 512, 384, 6, 102), ("bf16", 520, 256, 132, 4, 101), ("bf16", 1000, 1024, 192, 4, 108)])
def test_route_gemm_and_selection(dtype, T, d, E, k, split):
    """router GEMM + selection; split: the few-token router's parts of K (-1 the library's choice, 0 the fused
    kernel, n forced; T = 700 is above the few-token limit and always fused).  From 16384 tokens on a workgroup
    takes 64 tokens, from 32768 on (up to 128 experts) 128: three cases with ragged last tiles.  With more than 128
    experts and enough tokens the logits come from the 256 x 256 GEMM tile with K in parts
    (T = 12300, d = 2560: 49 token tiles, the last with 12 tokens, and the library takes 5 parts of 8 slices = 245
    workgroups; where tiles x parts would fill less than three quarters of the compute units it stays with the fused
    kernel); 100 + n forces that form with n
    parts: ragged token tiles, a second expert tile half filled (E = 384), E not a multiple of 32, two slices a part"""
    _say("route", dtype, T, d, E, k, "split", split)
    w = WL.small(T=T, d=d, E=E, k=k, D=1, C=4, dtype=dtype)
    inp = H.make_inputs(w)
    lay = H.Layer(w)
    b_g = (0.1 * np.random.default_rng(1).standard_normal(E)).astype(np.float32)
    lay.m.set_tuning(7, split)
    try:
        logits, ids, tw = lay.route(inp, b_g=b_g)
    finally:
        lay.m.set_tuning(7, -1)
    want_logits = O.route_logits(inp.X, inp.W_r, b_g, inp.token_class, inp.class_bias)
    err = O.max_rel_err(logits, want_logits)
    assert err <= 1e-5, err              # inputs are exact in both; only fp32 accumulation order differs
    want_ids, want_w = H.oracle_select(w, logits)
    assert (ids == want_ids).all()
    assert O.max_rel_err(tw, want_w) <= 1e-5
    _say("  logits err %.2e, ids that differ from the oracle-logits selection: %.4f" %
         (err, (want_ids != H.oracle_select(w, want_logits)[0]).any(axis=1).mean()))


# ------------------------------------------------------------------------------------------- coact_hist
@pytest.mark.parametrize("T,E,k", [(1000, 16, 2), (5000, 128, 8), (777, 256, 8), (300, 512, 16), (64, 8, 1)])
def test_coact_hist_bit_exact_and_accumulating(T, E, k):
    _say("coact_hist", T, E, k)
    ids = WL.uniform_random_ids(T, E, k, seed=T)
    m = S.SemMoE(S.Config(T=T, d=8, E=E, k=k, F=8, D=1, cap=T), allocate_workspace=False)
    load = torch.zeros(E, dtype=torch.int32, device=H.DEV)
    co = torch.zeros(E, E, dtype=torch.int32, device=H.DEV)
    ids_d = H.to_dev(ids)
    half = T // 3
    m.coact_hist(ids_d[:half].contiguous(), half, load, co)
    m.coact_hist(ids_d[half:].contiguous(), T - half, load, co)
    torch.cuda.synchronize()
    wl, wc = O.coact_hist(ids, E)
    assert (H.to_np(load) == wl).all() and (H.to_np(co) == wc).all()


# ------------------------------------------------------------------------------------------- reshuffle
def _planted(T, E, D, k, seed, noise):
    r = np.random.default_rng(seed)
    m = E // D
    e2r = r.permutation(np.repeat(np.arange(D), m)).astype(np.int32)
    members = [np.flatnonzero(e2r == c) for c in range(D)]
    p = (np.arange(D) + 1.0) ** -1.2
    p /= p.sum()
    ids = np.zeros((T, k), dtype=np.int32)
    for i in range(T):
        if r.random() < noise or k > m:
            ids[i] = r.choice(E, k, replace=False)
        else:
            c = r.choice(D, p=p)                      # skewed: capacity binds on the popular ranks
            ids[i] = r.choice(members[c], k, replace=False)
    return ids, e2r


@pytest.mark.parametrize("T,E,D,k,cf,noise", [
    (256, 16, 4, 2, 1.0, 0.2), (1000, 128, 8, 8, 1.0, 0.5), (777, 64, 16, 4, 1.0, 0.3), (300, 32, 32, 2, 1.0, 0.5),
    (513, 16, 4, 4, 1.25, 0.4), (100, 8, 1, 2, 1.0, 0.5), (2049, 64, 64, 1, 1.0, 0.0), (64, 16, 8, 2, 8.0, 0.3),
    (5, 16, 4, 2, 1.0, 0.5), (4000, 256, 32, 8, 1.0, 0.6)])
def test_reshuffle_bit_exact(T, E, D, k, cf, noise, index_path):
    _say("reshuffle", T, E, D, k, cf, "path", index_path)
    ids, e2r = _planted(T, E, D, k, seed=T + D, noise=noise)
    cap = int(math.ceil(cf * T / D))
    w = WL.small(T=T, E=E, D=D, k=k)
    lay = H.Layer(w, cap=cap)
    lay.set_routing(ids)
    lay.e2r = H.to_dev(e2r)
    got = lay.reshuffle()
    want = O.reshuffle(ids, e2r, D, cap)
    for g, w_, name in zip(got, want, ("token_rank", "shf", "inv_shf", "rank_count")):
        assert (g == w_).all(), name
    assert (got[3] <= cap).all()


@pytest.mark.parametrize("T,E,D,k,cf,noise", [
    (256, 16, 4, 2, 1.0, 0.2), (1000, 128, 8, 8, 1.0, 0.5), (777, 64, 16, 4, 1.0, 0.3), (300, 32, 32, 2, 1.0, 0.5),
    (513, 16, 4, 4, 1.25, 0.4), (100, 8, 1, 2, 1.0, 0.5), (2049, 64, 64, 1, 1.0, 0.0), (5, 16, 4, 2, 1.0, 0.5),
    (4000, 256, 32, 8, 1.0, 0.6), (3000, 48, 3, 16, 1.0, 0.1)])
@pytest.mark.parametrize("rounds", [1, 2, 3, 64])
def test_reshuffle_rounds_bit_exact(T, E, D, k, cf, noise, rounds):
    """gain-aware spill rounds against the oracle, bit for bit; rounds = 1 is also the plain reshuffle"""
    _say("reshuffle rounds", T, E, D, k, cf, "rounds", rounds)
    ids, e2r = _planted(T, E, D, k, seed=T + D, noise=noise)
    cap = int(math.ceil(cf * T / D))
    w = WL.small(T=T, E=E, D=D, k=k)
    lay = H.Layer(w, cap=cap)
    lay.set_routing(ids)
    lay.e2r = H.to_dev(e2r)
    got = lay.reshuffle_rounds(rounds)
    want = O.reshuffle_rounds(ids, e2r, D, cap, min(rounds, D))
    for g, w_, name in zip(got, want, ("token_rank", "shf", "inv_shf", "rank_count")):
        assert (g == w_).all(), (name, np.flatnonzero(g != w_)[:8])
    assert (got[3] <= cap).all()
    if rounds == 1:
        for g, w_ in zip(got, O.reshuffle(ids, e2r, D, cap)):
            assert (g == w_).all()


@pytest.mark.parametrize("T,E,D,k,cf,noise", [
    (256, 16, 4, 2, 1.0, 0.2), (1000, 128, 8, 8, 1.0, 0.5), (513, 16, 4, 4, 1.25, 0.4), (100, 8, 1, 2, 1.0, 0.5),
    (5, 16, 4, 2, 1.0, 0.5), (3000, 48, 3, 15, 1.0, 0.3), (777, 64, 8, 4, 1.0, 0.3), (8192, 64, 8, 4, 1.0, 0.4),
    (8193, 32, 4, 2, 1.0, 0.3), (20000, 128, 8, 8, 1.0, 0.6), (32768, 64, 8, 6, 1.0, 0.5), (700, 14, 7, 2, 1.1, 0.2),
    (900, 64, 16, 4, 1.0, 0.4), (3000, 36, 9, 4, 1.0, 0.3), (10000, 128, 16, 8, 1.0, 0.5), (20000, 60, 12, 5, 1.0, 0.4),
    (32768, 128, 16, 4, 1.0, 0.5), (400, 13, 13, 1, 1.0, 0.0)])
@pytest.mark.parametrize("rounds,max_cycles", [(1, 1 << 30), (3, 1 << 30), (1, 0), (1, 3)])
def test_reshuffle_refine_bit_exact(T, E, D, k, cf, noise, rounds, max_cycles):
    """moves of placed tokens until the assignment is optimal, against the oracle's cycle by cycle: same tokens,
    same number of cycles, same verdict; every form of the workgroup (8, 16, 32 tokens per thread; up to 8 and up to 16 ranks)"""
    _say("reshuffle refine", T, E, D, k, cf, "rounds", rounds, "max_cycles", max_cycles)
    ids, e2r = _planted(T, E, D, k, seed=T + D, noise=noise)
    cap = int(math.ceil(cf * T / D))
    w = WL.small(T=T, E=E, D=D, k=k)
    lay = H.Layer(w, cap=cap)
    lay.set_routing(ids)
    lay.e2r = H.to_dev(e2r)
    got, cycles, conv = lay.reshuffle_refine(rounds, max_cycles)
    want, wcycles, wconv = O.reshuffle_refine(ids, e2r, D, cap, max_cycles, rounds=min(rounds, D))
    assert (cycles, conv) == (wcycles, int(wconv))
    for g, w_, name in zip(got, want, ("token_rank", "shf", "inv_shf", "rank_count")):
        assert (g == w_).all(), (name, np.flatnonzero(g != w_)[:8])
    assert (got[3] <= cap).all()
    start = O.reshuffle_rounds(ids, e2r, D, cap, min(rounds, D))[0]
    assert O.local_pairs(ids, e2r, got[0]) >= O.local_pairs(ids, e2r, start) + cycles
    if max_cycles == 0:
        assert (got[0] == start).all()


def test_reshuffle_refine_reaches_the_min_cost_flow_optimum():
    """the end state against the exact optimum of the assignment problem (a different algorithm)"""
    _say("reshuffle refine vs min-cost flow")
    for T, E, D, k in ((160, 16, 4, 2), (200, 32, 8, 4)):
        ids, e2r = _planted(T, E, D, k, seed=3 * T, noise=0.3)
        cap = T // D
        lay = H.Layer(WL.small(T=T, E=E, D=D, k=k), cap=cap)
        lay.set_routing(ids)
        lay.e2r = H.to_dev(e2r)
        got, cycles, conv = lay.reshuffle_refine()
        assert conv == 1
        assert O.local_pairs(ids, e2r, got[0]) == O.reshuffle_exact(ids, e2r, D, cap)[1]


def test_reshuffle_refine_refuses_what_one_workgroup_cannot_hold():
    lay = H.Layer(WL.small(T=64, E=64, D=32, k=2), cap=2)
    i32 = dict(dtype=torch.int32, device=H.DEV)
    one = torch.zeros(256, **i32)
    with pytest.raises(Exception) as ei:
        lay.m.reshuffle_refine(one, one, 1, 10, one, one, one, one, one, cap=2)
    assert getattr(ei.value, "status", None) == -5


@pytest.mark.parametrize("T,E,D,k,V,batches", [
    (256, 16, 4, 2, 64, 1), (1000, 128, 8, 8, 500, 3), (777, 64, 16, 4, 33, 2), (5, 16, 4, 2, 7, 1),
    (4000, 256, 32, 8, 1000, 2), (3000, 48, 3, 16, 128, 1), (70000, 32, 4, 2, 9, 1)])
def test_token_expert_hist_bit_exact(T, E, D, k, V, batches):
    """token-to-expert activation table against the oracle, accumulated over batches; pairs whose key lies outside
    the vocabulary or whose expert id lies outside [0,E) are skipped (the oracle is given the valid pairs only)"""
    _say("token-expert hist", T, E, D, k, V, batches)
    r = np.random.default_rng(T * 3 + V)
    lay = H.Layer(WL.small(T=T, E=E, D=D, k=k, d=8))
    table, want = None, None
    for b in range(batches):
        ids, _ = _planted(T, E, D, k, seed=T + b, noise=0.4)
        keys = r.integers(0, V, size=T).astype(np.int32)
        if b == batches - 1 and T > 4:
            keys[1], keys[2] = V + 5, -1
            ids[3, 0], ids[4, k - 1] = -1, E
        pair_key = np.repeat(keys, k)
        pair_id = ids.reshape(-1, 1)
        ok = (pair_key >= 0) & (pair_key < V) & (pair_id[:, 0] >= 0) & (pair_id[:, 0] < E)
        want = O.token_expert_table(pair_key[ok], pair_id[ok], V, E, want)
        table = lay.token_expert_hist(keys, ids, V, table)
    got = H.to_np(table).astype(np.int64)
    assert (got == want).all(), np.argwhere(got != want)[:8]


@pytest.mark.parametrize("T,E,D,k,cf,V,thr", [
    (256, 16, 4, 2, 1.0, 64, 0), (1000, 128, 8, 8, 1.0, 200, 20000), (777, 64, 16, 4, 1.0, 33, 30000),
    (300, 32, 32, 2, 1.0, 100, 0), (513, 16, 4, 4, 1.25, 50, 40000), (100, 8, 1, 2, 1.0, 10, 0),
    (2049, 64, 64, 1, 1.0, 300, 10000), (5, 16, 4, 2, 1.0, 4, 0), (4000, 256, 32, 8, 1.0, 700, 16384),
    (3000, 48, 3, 16, 1.0, 256, 65536), (3000, 48, 3, 16, 1.0, 256, -1), (40000, 64, 16, 4, 1.0, 320, 20000)])
def test_reshuffle_lookup_bit_exact(T, E, D, k, cf, V, thr):
    """table-driven reshuffle against the oracle, bit for bit: the tables come from the library's own profile pass
    (device histogram, host tables), checked against the oracle's, then one rebatch from keys alone; a few keys
    are left unseen and a few lie outside the table"""
    _say("reshuffle lookup", T, E, D, k, cf, V, thr)
    r = np.random.default_rng(T + V)
    ids, e2r = _planted(T, E, D, k, seed=T + D, noise=0.3)
    # keys follow the planted cluster of the token, so that the table predicts: cluster c owns keys = c mod D
    g = O.gain_matrix(ids, e2r, D)
    keys = (g.argmax(axis=1) + D * r.integers(0, max(V // D, 1), size=T)).astype(np.int32) % V
    seen = r.random(T) < 0.9                      # profile on most tokens only: some keys stay unseen
    cap = int(math.ceil(cf * T / D))
    w = WL.small(T=T, E=E, D=D, k=k)
    lay = H.Layer(w, cap=cap)
    table = H.to_np(lay.token_expert_hist(keys[seen], ids[seen], V)).astype(np.int64)
    assert (table == O.token_expert_table(keys[seen], ids[seen], V, E)).all()
    dev, conf, level = lay.m.lookup_tables(table.astype(np.uint32), e2r)
    for g_, w_ in zip((dev, conf, level), O.lookup_tables(table, e2r, D, k)):
        assert (g_ == w_).all()
    got = lay.reshuffle_lookup(keys, dev, conf, level, thr, cap=cap)
    want = O.reshuffle_lookup(keys, dev, conf, level, thr, D, cap)
    for g_, w_, name in zip(got, want, ("token_rank", "shf", "inv_shf", "rank_count")):
        assert (g_ == w_).all(), (name, np.flatnonzero(g_ != w_)[:8])
    assert (got[3] <= cap).all()
    if thr >= 65536:                               # 65536 = certainty: nothing exceeds it, everyone stays home
        assert (got[0] == O.home_rank(T, D)).all()
    if T > 8:                                      # keys outside the table stay home with priority 0
        keys2 = keys.copy()
        keys2[::7] = V + 3
        keys2[3::7] = -2
        dev2 = np.concatenate([dev, [-1]]).astype(np.int32)       # the oracle reads them as one more unseen key
        conf2 = np.concatenate([conf, [0]]).astype(np.int32)
        lev2 = np.concatenate([level, [0]]).astype(np.int32)
        kk = np.where((keys2 < 0) | (keys2 >= V), V, keys2)
        got2 = lay.reshuffle_lookup(keys2, dev, conf, level, thr, cap=cap)
        want2 = O.reshuffle_lookup(kk, dev2, conf2, lev2, thr, D, cap)
        for g_, w_ in zip(got2, want2):
            assert (g_ == w_).all()


@pytest.mark.parametrize("T,E,D,k", [(256, 16, 4, 2), (1000, 128, 8, 8), (777, 64, 16, 4), (300, 32, 32, 2),
                                     (5, 16, 4, 2), (3000, 48, 3, 16), (40000, 64, 16, 4), (513, 8, 8, 1)])
def test_device_sequence_bit_exact(T, E, D, k):
    """the device a token selects (most of its k experts, equal -> smallest), alone and chained over two layers
    with unknown histories in between"""
    _say("device sequence", T, E, D, k)
    r = np.random.default_rng(T + E)
    ids, e2r = _planted(T, E, D, k, seed=T + D, noise=0.5)
    ids2, e2r2 = _planted(T, E, D, k, seed=T + D + 1, noise=0.5)
    lay = H.Layer(WL.small(T=T, E=E, D=D, k=k))
    one = lay.device_sequence(ids, e2r)
    assert (one == O.device_sequence(ids, e2r, D)).all()
    prev = one.copy()
    prev[r.random(T) < 0.1] = -1
    two = lay.device_sequence(ids2, e2r2, prev)
    assert (two == O.device_sequence(ids2, e2r2, D, prev)).all()
    assert ((two == -1) == (prev == -1)).all() and two.max() < D * D


@pytest.mark.parametrize("T,E,D,k,cf,V,thr", [
    (256, 16, 4, 2, 1.0, 64, -1), (1000, 128, 8, 8, 1.0, 200, 20000), (777, 64, 16, 4, 1.0, 33, 30000),
    (300, 32, 32, 2, 1.0, 100, 0), (513, 16, 4, 4, 1.25, 50, 40000), (100, 8, 1, 2, 1.0, 10, 0),
    (2049, 64, 64, 1, 1.0, 300, 10000), (5, 16, 4, 2, 1.0, 4, -1), (4000, 256, 32, 8, 1.0, 700, 16384),
    (3000, 48, 3, 16, 1.0, 256, 65536), (40000, 64, 16, 4, 1.0, 320, -1)])
def test_reshuffle_cond_bit_exact(T, E, D, k, cf, V, thr):
    """Alg. 3 with both tables against the oracle, bit for bit.  Both tables come from the library's own profile
    pass: T keyed by token keys of which a third say nothing about the token's cluster, A keyed by the device
    sequence of two earlier layers (library kernel), some histories unknown, some keys outside the table"""
    _say("reshuffle cond", T, E, D, k, cf, V, thr)
    r = np.random.default_rng(T + V + 1)
    ids, e2r = _planted(T, E, D, k, seed=T + D, noise=0.3)
    g = O.gain_matrix(ids, e2r, D).argmax(axis=1)
    keys = (g + D * r.integers(0, max(V // D, 1), size=T)).astype(np.int32) % V
    vague = r.random(T) < 0.33
    keys[vague] = r.integers(0, V, size=int(vague.sum()))
    cap = int(math.ceil(cf * T / D))
    lay = H.Layer(WL.small(T=T, E=E, D=D, k=k), cap=cap)
    # two earlier layers whose routing follows the same clusters with other noise
    prev = None
    for layer in (2, 1):
        ids_l = ids.copy()
        flip = r.random(T) < 0.3
        ids_l[flip] = _planted(T, E, D, k, seed=T + D + layer, noise=1.0)[0][flip]
        prev = lay.device_sequence(ids_l, e2r, prev)
    seq = prev.copy()
    seq[r.random(T) < 0.05] = -1
    VA = D * D
    seen = r.random(T) < 0.9
    tab_t = H.to_np(lay.token_expert_hist(keys[seen], ids[seen], V)).astype(np.uint32)
    ok = seen & (seq >= 0)
    tab_a = H.to_np(lay.token_expert_hist(seq[ok], ids[ok], VA)).astype(np.uint32)
    tt = lay.m.lookup_tables(tab_t, e2r)
    ta = lay.m.lookup_tables(tab_a, e2r)
    keys2 = keys.copy()
    if T > 8:
        keys2[::11] = V + 3
        keys2[5::11] = -2
    got = lay.reshuffle_cond(keys2, tt, seq, ta, thr, cap=cap)
    want = O.reshuffle_cond(keys2, *tt, seq, *ta, thr, D, cap)
    for g_, w_, name in zip(got, want, ("token_rank", "shf", "inv_shf", "rank_count")):
        assert (g_ == w_).all(), (name, np.flatnonzero(g_ != w_)[:8])
    assert (got[3] <= cap).all()
    if thr >= 65536:
        assert (got[0] == O.home_rank(T, D)).all()
    # one table empty: the call equals the single-table entry point
    none = tuple(np.array(x, dtype=np.int32) for x in ([-1], [0], [0]))
    a = lay.reshuffle_cond(keys2, tt, seq, none, thr, cap=cap)
    b = lay.reshuffle_lookup(keys2, *tt, thr, cap=cap)
    for g_, w_ in zip(a, b):
        assert (g_ == w_).all()


@pytest.mark.parametrize("T,D,V,n_req,seed", [
    (256, 4, 64, 7, 0), (1000, 8, 500, 40, 1), (777, 16, 33, 100, 2), (5, 4, 7, 5, 3), (4000, 32, 1000, 64, 4),
    (3000, 3, 128, 1, 5), (2049, 64, 300, 200, 6), (100, 1, 10, 9, 7), (100000, 8, 1088, 3000, 8),
    (64, 8, 16, 64, 9)])
def test_request_schedule_bit_exact(T, D, V, n_req, seed):
    """request-level scheduling against the oracle, bit for bit: ranks of the requests, the tokens' ranks and the
    shuffle; random request lengths with empty requests, a table with unseen keys, keys outside the table"""
    _say("request schedule", T, D, V, n_req, seed)
    r = np.random.default_rng(seed)
    cuts = np.sort(r.integers(0, T + 1, size=n_req - 1)) if n_req > 1 else np.zeros(0, dtype=np.int64)
    if n_req == T:
        cuts = np.arange(1, T)                      # one token per request
    off = np.concatenate([[0], cuts, [T]]).astype(np.int32)
    dev = r.integers(-1, D, size=V).astype(np.int32)
    # requests lean towards one device each, so that the mask decides often
    keys = r.integers(0, V, size=T).astype(np.int32)
    by_dev = [np.flatnonzero(dev == x) for x in range(D)]
    for q in range(n_req):
        x = int(r.integers(0, D))
        if len(by_dev[x]) and off[q + 1] > off[q]:
            lean = r.random(off[q + 1] - off[q]) < 0.6
            keys[off[q]:off[q + 1]][lean] = r.choice(by_dev[x], size=int(lean.sum()))
    lay = H.Layer(WL.small(T=T, E=2 * D, D=D, k=1, d=8))
    got = lay.request_schedule(off, keys, dev)
    want_rr = O.request_schedule(off, keys, dev, D)
    want = (want_rr,) + O.request_assignment(off, want_rr, D)
    for g, w_, name in zip(got, want, ("req_rank", "token_rank", "shf", "inv_shf", "rank_count")):
        assert (g == w_).all(), (name, np.flatnonzero(g != w_)[:8])
    if T > 8:                                       # keys outside the table count nowhere
        keys2 = keys.copy()
        keys2[::5] = V + 1
        keys2[2::5] = -3
        dev2 = np.concatenate([dev, [-1]]).astype(np.int32)
        kk = np.where((keys2 < 0) | (keys2 >= V), V, keys2)
        got2 = lay.request_schedule(off, keys2, dev)
        want_rr2 = O.request_schedule(off, kk, dev2, D)
        want2 = (want_rr2,) + O.request_assignment(off, want_rr2, D)
        for g, w_ in zip(got2, want2):
            assert (g == w_).all()


@pytest.mark.parametrize("T,E,D,k", [(40000, 64, 16, 4), (131072, 8, 4, 2), (131073, 8, 4, 2)])
def test_reshuffle_and_dispatch_index_above_the_single_workgroup_limit(T, E, D, k):
    """beyond what the single-workgroup kernels hold; multi-workgroup kernels by default.  T = 131072 is the last
    size of the two-launch kernels (512 workgroups read the whole count table), one token more takes the kernels
    with scan launches in between"""
    _say("reshuffle + dispatch index, large T", T)
    ids, e2r = _planted(T, E, D, k, seed=5, noise=0.4)
    phys = np.argsort(np.argsort(e2r, kind="stable"), kind="stable").astype(np.int32)
    w = WL.small(T=T, E=E, D=D, k=k, d=8)
    lay = H.Layer(w)
    lay.set_routing(ids)
    lay.set_placement(e2r, phys, np.argsort(phys).astype(np.int32))
    got = lay.reshuffle()
    want = O.reshuffle(ids, e2r, D, w.cap)
    for g, w_ in zip(got, want):
        assert (g == w_).all()
    lay.X = None
    dg = lay.dispatch(with_rows=False)
    dw = O.dispatch(None, ids, want[0], want[2], phys, D)
    for name in ("slot_of_pair", "pair_of_slot", "expert_offsets", "rank_offsets", "send_matrix"):
        assert (dg[name] == dw[name]).all(), name


@pytest.mark.parametrize("seed", list(range(12)))
def test_index_kernels_on_random_shapes(seed, index_path):
    """reshuffle + dispatch index on seeded random shapes (ragged T, D up to 64, k up to 16, tight and loose
    capacity, clustered and noisy routing), every implementation of the index kernels, bit for bit"""
    r = np.random.default_rng(1000 + seed)
    D = int(r.choice([1, 2, 4, 8, 16, 32, 64]))
    m = int(r.choice([1, 2, 4, 8]))
    E = D * m
    k = int(min(E, r.choice([1, 2, 4, 8, 16])))
    T = int(r.integers(1, 6000))
    cf = float(r.choice([1.0, 1.0, 1.1, 2.0]))
    noise = float(r.choice([0.0, 0.2, 0.6, 1.0]))
    _say("index kernels, random shape", dict(T=T, E=E, D=D, k=k, cf=cf, noise=noise), "path", index_path)
    ids, e2r = _planted(T, E, D, k, seed=seed, noise=noise)
    phys = np.argsort(np.argsort(e2r, kind="stable"), kind="stable").astype(np.int32)
    cap = int(math.ceil(cf * T / D))
    w = WL.small(T=T, E=E, D=D, k=k, d=8)
    lay = H.Layer(w, cap=cap)
    lay.set_routing(ids)
    lay.set_placement(e2r, phys, np.argsort(phys).astype(np.int32))
    got = lay.reshuffle()
    want = O.reshuffle(ids, e2r, D, cap)
    for g, w_, name in zip(got, want, ("token_rank", "shf", "inv_shf", "rank_count")):
        assert (g == w_).all(), name
    dg = lay.dispatch(with_rows=False)
    dw = O.dispatch(None, ids, want[0], want[2], phys, D)
    for name in ("slot_of_pair", "pair_of_slot", "expert_offsets", "rank_offsets", "send_matrix"):
        assert (dg[name] == dw[name]).all(), name
    assert int(dg["remote_pairs"]) == int(dw["remote_pairs"])


# ------------------------------------------------------------------------------------------- dispatch
@pytest.mark.parametrize("dtype,T,E,D,k,d", [("bf16", 700, 128, 8, 8, 64), ("fp32", 256, 16, 4, 2, 40),
                                              ("bf16", 1030, 256, 32, 8, 136), ("bf16", 90, 8, 2, 1, 8),
                                              ("fp32", 300, 24, 3, 3, 16), ("bf16", 513, 512, 64, 16, 24)])
def test_dispatch_bit_exact(dtype, T, E, D, k, d, index_path):
    _say("dispatch", dtype, T, E, D, k, d, "path", index_path)
    w = WL.small(T=T, E=E, D=D, k=k, d=d, dtype=dtype)
    ids, e2r = _planted(T, E, D, k, seed=T, noise=0.4)
    m = E // D
    phys = np.zeros(E, dtype=np.int32)
    seen = [0] * D
    for e in range(E):
        phys[e] = e2r[e] * m + seen[e2r[e]]
        seen[e2r[e]] += 1
    inv = np.argsort(phys).astype(np.int32)
    tr, shf, ishf, rc = O.reshuffle(ids, e2r, D, w.cap)
    lay = H.Layer(w)
    lay.X = H.to_dev(WL.hidden(w), w)
    lay.set_routing(ids)
    lay.set_placement(e2r, phys, inv)
    lay.set_assignment(tr, shf, ishf)
    got = lay.dispatch()
    want = O.dispatch(WL.hidden(w), ids, tr, ishf, phys, D)
    for name in ("slot_of_pair", "pair_of_slot", "expert_offsets", "rank_offsets", "send_matrix"):
        assert (got[name] == want[name]).all(), name
    assert int(got["remote_pairs"]) == int(want["remote_pairs"])
    assert (H.to_np(lay.X_perm) == want["X_perm"]).all()          # rows are bit copies
    assert sorted(got["slot_of_pair"]) == list(range(T * k))      # every pair dispatched exactly once


# ------------------------------------------------------------------------------------------- FFN + combine + whole path
def _run_path(w, placed=True, shuffle=True, cf=1.0, rank=-1, shared=False):
    inp = H.make_inputs(w)
    cap = int(math.ceil(cf * w.T / w.D))
    lay = H.Layer(w, cap=cap)
    logits, ids, tw = lay.route(inp)
    want_ids, want_w = H.oracle_select(w, logits)
    assert (ids == want_ids).all()
    # placement from a separate profiling batch, through coact_hist + the host solver
    if placed:
        pinp = H.make_inputs(w, profile=True)
        play = H.Layer(w, T=pinp.X.shape[0])
        plog, pids, _ = play.route(pinp)
        load, co, (e2r, phys, inv) = play.profile_placement(play.ids)
        ol, oc = O.coact_hist(pids, w.E)
        assert (load == ol).all() and (co == oc).all()
        oe2r, ophys, oinv = O.place(ol, oc, w.D)
        assert (e2r == oe2r).all() and (phys == ophys).all() and (inv == oinv).all()
    else:
        e2r, phys, inv = O.vanilla_placement(w.E, w.D)
    lay.set_placement(e2r, phys, inv)
    if shuffle:
        got = lay.reshuffle()
        want = O.reshuffle(ids, e2r, w.D, cap)
        for g, w_ in zip(got, want):
            assert (g == w_).all()
        tr, shf, ishf, rc = want
    else:
        tr, shf, ishf, rc = O.home_assignment(w.T, w.D)
        lay.set_assignment(tr, shf, ishf)
    dg = lay.dispatch()
    dw = O.dispatch(inp.X, ids, tr, ishf, phys, w.D)
    for name in ("slot_of_pair", "pair_of_slot", "expert_offsets", "rank_offsets", "send_matrix"):
        assert (dg[name] == dw[name]).all(), name
    assert (H.to_np(lay.X_perm) == dw["X_perm"]).all()
    weights = {e: WL.expert_weight(w, e) for e in range(w.E)}
    lay.load_experts(range(w.E))
    Y = H.to_np(lay.expert_ffn(rank, poison=512.0))
    Yo = O.expert_ffn(dw["X_perm"], dw["expert_offsets"], inv, lambda e: weights[e], w.D, rank=rank,
                      Y=np.full(Y.shape, 512.0))
    return lay, inp, ids, want_w, dw, Y, Yo, weights


@pytest.mark.parametrize("dtype,T,d,E,k,F,D,rank", [
    ("bf16", 200, 64, 16, 2, 96, 4, -1), ("bf16", 700, 200, 32, 4, 72, 4, 1), ("fp32", 150, 72, 16, 2, 40, 4, -1),
    ("bf16", 1300, 136, 8, 2, 264, 2, 0), ("fp32", 300, 64, 8, 3, 104, 2, 1), ("bf16", 64, 128, 64, 8, 128, 8, -1)])
def test_expert_ffn_and_combine(dtype, T, d, E, k, F, D, rank):
    _say("ffn+combine", dtype, T, d, E, k, F, D, rank)
    w = WL.small(T=T, d=d, E=E, k=k, F=F, D=D, dtype=dtype, C=D)
    lay, inp, ids, want_w, dw, Y, Yo, weights = _run_path(w, rank=rank)
    lo, hi = (0, T * k) if rank < 0 else (dw["rank_offsets"][rank], dw["rank_offsets"][rank + 1])
    assert (Y[:lo] == 512.0).all() and (Y[hi:] == 512.0).all()          # other ranks' rows untouched
    if hi > lo:
        H.assert_close(Y[lo:hi], Yo[lo:hi], dtype, "Y")
    if rank < 0:
        out = lay.combine()
        H.assert_close(out, O.combine(Yo, dw["slot_of_pair"], want_w), dtype, "Out (oracle chain)")
        ref = O.moe_definition(inp.X, ids, want_w, lambda e: weights[e])
        H.assert_close(out, ref, dtype, "Out vs plain MoE definition")


@pytest.mark.parametrize("placed,shuffle,cf", [(False, False, 1.0), (True, False, 1.0), (True, True, 1.0),
                                               (True, True, 1.5)])
def test_layer_output_is_independent_of_placement_and_shuffle(placed, shuffle, cf):
    """lossless (Sec. 5): all variants equal the plain MoE definition"""
    _say("lossless", placed, shuffle, cf)
    w = WL.small(T=300, d=64, E=16, k=2, F=64, D=4, dtype="bf16", n_shared=1)
    lay, inp, ids, want_w, dw, Y, Yo, weights = _run_path(w, placed, shuffle, cf)
    ysh = lay.shared_ffn()
    out = lay.combine(Y_shared=ysh)
    shared = WL.shared_weight(w)
    H.assert_close(H.to_np(ysh), O.swiglu_ffn(inp.X, *shared), "bf16", "Y_shared")
    ref = O.moe_definition(inp.X, ids, want_w, lambda e: weights[e], shared)
    H.assert_close(out, ref, "bf16", "Out")


@pytest.mark.parametrize("dtype,k", [("bf16", 1), ("bf16", 2), ("bf16", 4), ("bf16", 8), ("fp32", 1), ("fp32", 2),
                                     ("bf16", 3), ("bf16", 6), ("bf16", 16), ("fp32", 5), ("fp32", 12)])
def test_combine_after_dispatch_is_identity_for_unit_weights(dtype, k):
    _say("combine identity", dtype, k)
    T, E, D, d = 500, 16, 4, 72
    w = WL.small(T=T, E=E, D=D, k=k, d=d, dtype=dtype)
    ids, e2r = _planted(T, E, D, k, seed=k, noise=0.5)
    phys = np.argsort(np.argsort(e2r, kind="stable"), kind="stable").astype(np.int32)
    tr, shf, ishf, rc = O.reshuffle(ids, e2r, D, w.cap)
    lay = H.Layer(w)
    X = WL.hidden(w)
    lay.X = H.to_dev(X, w)
    lay.set_routing(ids, np.ones((T, k), dtype=np.float32))
    lay.set_placement(e2r, phys, np.argsort(phys).astype(np.int32))
    lay.set_assignment(tr, shf, ishf)
    lay.dispatch()
    out = lay.combine(Y=lay.X_perm)
    if k in (1, 2, 4, 8):
        assert (out == k * X).all()                   # exact: power-of-two scaling
    else:
        H.assert_close(out, k * X.astype(np.float64), dtype, "k*X")
    onehot = np.zeros((T, k), dtype=np.float32)
    onehot[:, k - 1] = 1
    lay.set_routing(ids, onehot)
    assert (lay.combine(Y=lay.X_perm) == X).all()


def test_combine_weights_and_shared_term():
    _say("combine weights")
    T, k, d = 260, 4, 136
    w = WL.small(T=T, k=k, d=d, dtype="bf16")
    r = np.random.default_rng(0)
    Y = WL.round_to_bf16(r.standard_normal((T * k, d)).astype(np.float32))
    Ysh = WL.round_to_bf16(r.standard_normal((T, d)).astype(np.float32))
    slot = r.permutation(T * k).astype(np.int32)
    tw = r.random((T, k)).astype(np.float32)
    lay = H.Layer(w)
    lay.slot_of_pair.copy_(torch.from_numpy(slot))
    lay.tw.copy_(torch.from_numpy(tw))
    out = lay.combine(Y=H.to_dev(Y, w), Y_shared=H.to_dev(Ysh, w))
    H.assert_close(out, O.combine(Y, slot, tw, Ysh), "bf16", "Out")


def test_empty_and_degenerate_inputs():
    _say("empty inputs")
    # T = 0: every call is a no-op that still returns OK
    w = WL.small(T=0, E=16, D=4, k=2)
    lay = H.Layer(w, cap=0)
    lay.e2r = H.to_dev(np.zeros(16, dtype=np.int32))
    lay.phys = H.to_dev(np.arange(16, dtype=np.int32))
    lay.inv = H.to_dev(np.arange(16, dtype=np.int32))
    tr, shf, ishf, rc = lay.reshuffle()
    assert (rc == 0).all()
    lay.X = torch.empty(0, w.d, dtype=torch.bfloat16, device=H.DEV)
    got = lay.dispatch()
    assert (got["expert_offsets"] == 0).all() and (got["rank_offsets"] == 0).all() and int(got["remote_pairs"]) == 0
    # the widened rows on an empty batch
    i32 = dict(dtype=torch.int32, device=H.DEV)
    rc_d = torch.full((4,), 7, **i32)
    one = torch.zeros(8, **i32)
    lay.m.reshuffle_rounds(one, lay.e2r, 3, one, one, one, rc_d, cap=0)
    torch.cuda.synchronize()
    assert (H.to_np(rc_d) == 0).all()
    rc_d.fill_(7)
    info = torch.full((2,), 9, **i32)
    lay.m.reshuffle_refine(one, lay.e2r, 1, 10, one, one, one, rc_d, info, cap=0)
    torch.cuda.synchronize()
    assert (H.to_np(rc_d) == 0).all() and (H.to_np(info) == 0).all()
    rc_d.fill_(7)
    lay.m.reshuffle_lookup(one, 8, one, one, one, 0, one, one, one, rc_d, cap=0)
    torch.cuda.synchronize()
    assert (H.to_np(rc_d) == 0).all()
    rc_d.fill_(7)
    lay.m.reshuffle_cond(one, 8, one, one, one, one, 8, one, one, one, 0, one, one, one, rc_d, cap=0)
    torch.cuda.synchronize()
    assert (H.to_np(rc_d) == 0).all()
    seq = torch.full((8,), 5, **i32)
    lay.m.device_sequence(one, lay.e2r, 0, None, seq)                           # no token: nothing written
    torch.cuda.synchronize()
    assert (H.to_np(seq) == 5).all()
    rc_d.fill_(7)
    lay.m.request_schedule(one, 0, one, 8, one, one, one, one, one, rc_d)       # no request, no token
    torch.cuda.synchronize()
    assert (H.to_np(rc_d) == 0).all()
    rc_d.fill_(7)
    rr = torch.full((1,), -5, **i32)
    lay.m.request_schedule(one, 1, one, 8, one, rr, one, one, one, rc_d)        # one empty request
    torch.cuda.synchronize()
    assert (H.to_np(rc_d) == 0).all() and H.to_np(rr).tolist() == [0]
    table = torch.zeros(8, 16, **i32)
    lay.m.token_expert_hist(one, one, 0, 8, table)
    torch.cuda.synchronize()
    assert int(table.sum().item()) == 0
    # an expert with zero rows writes nothing; all tokens on one expert pair
    w = WL.small(T=130, E=8, D=2, k=2, d=64, F=64)
    ids = np.tile(np.array([[3, 5]], dtype=np.int32), (130, 1))
    e2r, phys, inv = O.vanilla_placement(8, 2)
    lay = H.Layer(w)
    lay.X = H.to_dev(WL.hidden(w), w)
    lay.set_routing(ids, np.full((130, 2), 0.5, dtype=np.float32))
    lay.set_placement(e2r, phys, inv)
    got = lay.reshuffle()
    want = O.reshuffle(ids, e2r, 2, w.cap)
    for g, w_ in zip(got, want):
        assert (g == w_).all()
    dg = lay.dispatch()
    assert list(np.diff(dg["expert_offsets"])) == [0, 0, 0, 130, 0, 130, 0, 0]
    lay.load_experts([3, 5])
    Y = H.to_np(lay.expert_ffn(-1, poison=1.0))
    weights = {e: WL.expert_weight(w, e) for e in (3, 5)}
    dw = O.dispatch(WL.hidden(w), ids, want[0], want[2], phys, 2)
    Yo = O.expert_ffn(dw["X_perm"], dw["expert_offsets"], inv, lambda e: weights[e], 2)
    H.assert_close(Y, Yo, "bf16", "Y")


@pytest.mark.parametrize("tile", [0, 3, 4, 6, 11, 12, 14, 15, 16, 17, 18, 19, 25, 26, 27, 28])
def test_every_gemm_tile_shape_on_a_ragged_problem(tile):
    """each tile shape of the bf16 grouped GEMMs (register-staged, direct-to-LDS ring, skinny), with ragged
    groups, partial K slices (d % 64 = 8, F % 32 = 8) and partial feature tiles"""
    _say("gemm tile", tile)
    w = WL.small(T=700, d=200, E=8, k=2, F=72, D=2, dtype="bf16", C=2)
    m = S.SemMoE(S.Config.from_workload(w), allocate_workspace=False)
    try:
        m.set_tuning(0, tile)
        m.set_tuning(1, tile)
        lay, inp, ids, want_w, dw, Y, Yo, weights = _run_path(w, rank=-1)
        H.assert_close(Y, Yo, "bf16", "Y")
        out = lay.combine()
        H.assert_close(out, O.moe_definition(inp.X, ids, want_w, lambda e: weights[e]), "bf16", "Out")
    finally:
        m.set_tuning(0, -1)
        m.set_tuning(1, -1)


@pytest.mark.parametrize("tile,grid_cap,split", [(20, -1, -1), (21, -1, -1), (22, -1, -1), (16, -1, -1), (20, 3, -1),
                                                 (28, -1, -1), (28, 3, -1),
                                                 (22, 5, -1), (21, 1, 0), (16, 7, -1), (22, 4, 0), (16, 2, 0),
                                                 (22, 1, 16), (20, 6, 3)])
def test_big_gemm_tiles_with_many_tiles_per_workgroup(tile, grid_cap, split):
    """the 256 x 256 kernels: groups of several token tiles with a ragged last one, a partial feature tile
    (F = 192 against 128 per tile), K a multiple of 64; grid_cap: few workgroups, so that each walks many tiles
    and the load stream runs across tile boundaries; split: one launch, or full rounds of big tiles + the rest
    as quarter tiles"""
    _say("big gemm tile", tile, "grid cap", grid_cap, "split", split)
    w = WL.small(T=2500, d=256, E=4, k=2, F=192, D=2, dtype="bf16", C=2)
    m = S.SemMoE(S.Config.from_workload(w), allocate_workspace=False)
    try:
        m.set_tuning(0, tile)
        m.set_tuning(1, tile)
        m.set_tuning(4, grid_cap)
        m.set_tuning(5, split)
        lay, inp, ids, want_w, dw, Y, Yo, weights = _run_path(w, rank=-1)
        H.assert_close(Y, Yo, "bf16", "Y")
        out = lay.combine()
        H.assert_close(out, O.moe_definition(inp.X, ids, want_w, lambda e: weights[e]), "bf16", "Out")
    finally:
        for key in (0, 1, 4, 5):
            m.set_tuning(key, -1)


@pytest.mark.parametrize("grid_cap,split,ring", [(1, 16, 6), (4, 8, 6), (-1, 16, 6), (1, 16, 3), (-1, 8, 3),
                                                  (2, 16, -1), (-1, 16, -1), (1, 8, -1), (1, 16, 1), (-1, 8, 1)])
def test_tail_launch_kernels(grid_cap, split, ring):
    """the tail of a split GEMM: 128 x 128 pieces in the head's launch (default) or as a second launch (1), and the
    128 x 64 pieces with a ring of 3 or 6"""
    _say("tail ring", ring, "grid cap", grid_cap, "split", split)
    w = WL.small(T=2500, d=512, E=4, k=2, F=192, D=2, dtype="bf16", C=2)
    m = S.SemMoE(S.Config.from_workload(w), allocate_workspace=False)
    try:
        m.set_tuning(0, 22)
        m.set_tuning(1, 22)
        m.set_tuning(4, grid_cap)
        m.set_tuning(5, split)
        m.set_tuning(6, ring)
        lay, inp, ids, want_w, dw, Y, Yo, weights = _run_path(w, rank=-1)
        H.assert_close(Y, Yo, "bf16", "Y")
    finally:
        for key in (0, 1, 4, 5, 6):
            m.set_tuning(key, -1)


def _split_plan(rows_per_group, n_feat, feat_per_tile, grid, thr16=8):
    """the tile arithmetic of a split grouped GEMM, as the launcher and the kernel do it: 256-row token tiles per
    group x feature tiles, the head takes the full rounds of `grid` workgroups unless more than thr16/16 of a round
    is left over; returns (listed, head, left_over)"""
    listed = sum(-(-r // 256) for r in rows_per_group) * -(-n_feat // feat_per_tile)
    rem = listed % grid
    head = listed if 16 * rem > thr16 * grid else listed - rem
    return listed, head, listed - head


@pytest.mark.parametrize("ring", [-1, 2])
@pytest.mark.parametrize("rows", [(9 * 256 + 100, 7 * 256 - 30), (10 * 256, 6 * 256 + 100)])
def test_in_launch_tail_pieces_of_the_split_gemm(rows, ring):
    """The tail of the default split launch (tile 22): pieces of the left-over 256 x 256 tiles inside the head's
    launch.  The kernel takes 128 x 64 pieces (eight per parent tile) when twice the number of 128 x 128 pieces
    still fits the grid, else 128 x 128 pieces; with the tail knob at 2 always the latter.  The shape is chosen with
    the kernel's own arithmetic so that the 128 x 64 branch provably runs, in both GEMMs:
      two groups of 10 + 7 token tiles (the last one ragged: 226 or 100 rows, so with 100 rows two of the four
      64-token pieces of a parent tile lie outside the group and are skipped, one is partly filled);
      gate/up: F = 192 against 128 features per tile -> 2 feature tiles (the second half filled), K = d = 320 = 5 slices;
      down:    N = d = 320 against 256 per tile -> 2 feature tiles (the second a quarter filled), K = F = 192 = 3
               slices, the fewest the pieces' ring of 3 takes;
      either way 17 x 2 = 34 tiles on a grid capped at 16 workgroups: 2 full rounds = 32 tiles for the head
      (2/16 of a round is left over, below the threshold of 8/16), 2 parent tiles left over = 8 pieces of
      128 x 128, and 2 x 8 = 16 <= 16 workgroups -> sixteen 128 x 64 pieces."""
    _say("in-launch tail pieces", rows, "tail knob", ring)
    d, F, grid = 320, 192, 16
    for n_feat, per_tile in ((F, 128), (d, 256)):
        listed, head, left = _split_plan(rows, n_feat, per_tile, grid)
        assert (listed, head, left) == (34, 32, 2)
        assert left * 4 > 0 and left * 4 * 2 <= grid          # the kernel's condition for the 128 x 64 pieces
    T = sum(rows)
    w = WL.small(T=T, d=d, E=2, k=1, F=F, D=1, dtype="bf16", C=1)
    ids = np.repeat(np.arange(2, dtype=np.int32), rows)[:, None]
    r = np.random.default_rng(5)
    ids = ids[r.permutation(T)]                              # dispatch has to gather the groups
    e2r, phys, inv = O.vanilla_placement(2, 1)
    m = S.SemMoE(S.Config.from_workload(w), allocate_workspace=False)
    try:
        m.set_tuning(0, 22)      # the 256 x 256 tiles of the full-size workloads (so few rows would take pieces throughout)
        m.set_tuning(1, 22)
        m.set_tuning(4, grid)
        m.set_tuning(6, ring)
        lay = H.Layer(w)
        X = WL.hidden(w)
        lay.X = H.to_dev(X, w)
        lay.set_routing(ids, np.ones((T, 1), dtype=np.float32))
        lay.set_placement(e2r, phys, inv)
        tr, shf, ishf, rc = lay.reshuffle()
        dg = lay.dispatch()
        assert tuple(np.diff(dg["expert_offsets"])) == tuple(rows)
        dw = O.dispatch(X, ids, tr, ishf, phys, 1)
        weights = {e: WL.expert_weight(w, e) for e in range(2)}
        lay.load_experts(range(2))
        Y = H.to_np(lay.expert_ffn(0, poison=512.0))
        Yo = O.expert_ffn(dw["X_perm"], dw["expert_offsets"], inv, lambda e: weights[e], 1)
        assert not (Y == 512.0).all(axis=1).any()            # every row was written
        H.assert_close(Y, Yo, "bf16", "Y")
        # per-row check as well: the pieces' rows are few, a global maximum alone would be lenient for them
        lo = dw["expert_offsets"][1] + (len(range(0, rows[1], 256)) - 1) * 256
        H.assert_close(Y[lo:], Yo[lo:], "bf16", "Y rows of the left-over tiles")
    finally:
        for key in (0, 1, 4, 6):
            m.set_tuning(key, -1)


@pytest.mark.parametrize("n_rows,d,F", [(300, 256, 192), (512, 320, 256), (100, 192, 200)])
def test_shared_ffn_as_pieces(n_rows, d, F):
    """the shared expert on a shard of tokens: so few rows that 256 x 256 tiles could not fill the chip, so the library
    takes 128 x 128 pieces throughout, and 128 x 64 ones where twice as many still fit the grid (300 rows, F = 192:
    2 x 2 parent tiles = 16 pieces, 32 <= the grid of 32; the last 64-token piece holds 44 rows, the two after it none);
    F = 200 is no multiple of 64: the pieces' K loop does not take the down projection, the register-staged kernel does"""
    _say("shared ffn as pieces", n_rows, d, F)
    w = WL.small(T=max(n_rows, 512), d=d, E=4, k=1, F=F, D=1, dtype="bf16", C=1, n_shared=1)
    lay = H.Layer(w)
    X = WL.hidden(w)
    lay.X = H.to_dev(X, w)
    wgu, wdn = WL.shared_weight(w)
    ysh = torch.full((w.T, d), 512.0, dtype=torch.bfloat16, device=H.DEV)
    lay.m.shared_ffn(lay.X, n_rows, H.to_dev(wgu, w), H.to_dev(wdn, w), ysh)
    torch.cuda.synchronize()
    got = H.to_np(ysh)
    assert (got[n_rows:] == 512.0).all()                       # rows beyond the shard untouched
    want = O.swiglu_ffn(X[:n_rows], wgu, wdn)
    H.assert_close(got[:n_rows], want, "bf16", "Y_shared")
    if n_rows % 64:
        H.assert_close(got[n_rows - n_rows % 64:n_rows], want[n_rows - n_rows % 64:], "bf16", "rows of the partly filled piece")


def test_probes_copy_and_mfma_loop():
    """the two probes bench.py reads achievable rates from: the copy copies, the MFMA loop's checksum is the exact sum"""
    m = S.SemMoE(S.Config(T=1, d=8, E=2, k=1, F=8, D=1, cap=1), allocate_workspace=False)
    src = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device=H.DEV)
    dst = torch.zeros_like(src)
    m.probe_copy(dst, src, src.numel())
    words = torch.zeros(2048 * 256, dtype=torch.int32, device=H.DEV)
    ones = torch.ones(1 << 18, dtype=torch.int32, device=H.DEV)                 # 1 MiB = 64 chunks of 16 KB
    m.probe_stream(ones, ones.numel() * 4, 0, words)
    filled = torch.zeros(1 << 18, dtype=torch.int32, device=H.DEV)
    m.probe_stream(filled, filled.numel() * 4, 1, words[:1])                     # the write form never touches the sink
    torch.cuda.synchronize()
    assert int(words[:64 * 256].sum().item()) == (1 << 18) and int(words[64 * 256:].sum().item()) == 0
    f = filled.view(-1, 4)
    assert bool((f[:, 0] == 1).all()) and bool((f[:, 1] == 2).all()) and bool((f[:, 2] == 3).all())
    assert torch.equal(f[:, 3], torch.arange(64, device=H.DEV, dtype=torch.int32).repeat_interleave(1024))
    ops = torch.ones(256 * 1024, dtype=torch.bfloat16, device=H.DEV)
    sink = torch.zeros(256 * 256, dtype=torch.float32, device=H.DEV)
    flops = m.probe_mfma(ops, 3, sink)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert flops == 256 * 4 * 16 * 3 * 2.0 * 32 * 32 * 16
    # all-ones operands: every accumulator element is 16 per MFMA; a lane sums 16 tiles x 16 elements
    assert (H.to_np(sink) == 3 * 16.0 * 256).all()


@pytest.mark.parametrize("variant", list(range(8)))
def test_probe_tile_loop_checksum(variant):
    """the steady-state tile loop probe: on all-ones operands every MFMA adds 16 to each accumulator element, so a
    lane's checksum is (its accumulator elements) x 16 x 4 k-steps x slices, whatever parts of the loop are left out"""
    m = S.SemMoE(S.Config(T=1, d=8, E=2, k=1, F=8, D=1, cap=1), allocate_workspace=False)
    n_panels, row_bytes, n_slices = 96, 1024, 9
    panels = torch.ones(n_panels * 256 * row_bytes // 2, dtype=torch.bfloat16, device=H.DEV)
    sink = torch.zeros(256 * 512, dtype=torch.float32, device=H.DEV)
    flops = m.probe_tile_loop(panels, n_panels, row_bytes, variant, n_slices, sink)
    torch.cuda.synchronize()
    assert flops == 256 * 2.0 * 256 * 256 * 64 * n_slices
    threads = 256 if variant < 4 else 512
    elems = 256 if variant < 4 else 128                      # 4 x 4 or 4 x 2 tiles of 16 elements per lane
    got = H.to_np(sink)[:256 * threads]
    assert (got == elems * 16.0 * 4 * n_slices).all()
    # argument checks happen on the host: too few panels, rows that are not whole 128-byte slices, one slice
    with pytest.raises(S.SemMoEError):
        m.probe_tile_loop(panels, 95, row_bytes, variant, n_slices, sink)
    with pytest.raises(S.SemMoEError):
        m.probe_tile_loop(panels, n_panels, 192, variant, n_slices, sink)
    with pytest.raises(S.SemMoEError):
        m.probe_tile_loop(panels, n_panels, row_bytes, variant, 1, sink)


@pytest.mark.parametrize("seed", list(range(10)))
def test_whole_path_on_random_shapes_with_default_kernels(seed):
    """the whole layer on seeded random shapes with the library's own choice of kernels (tile shapes by rows per
    expert, split launches, fall-backs for K that the big tiles do not take), and a random cap on the GEMM grids so
    that the split between head and tail launches lands at different places"""
    r = np.random.default_rng(2000 + seed)
    D = int(r.choice([1, 2, 4]))
    E = D * int(r.choice([1, 2, 4]))
    k = int(min(E, r.choice([1, 2, 4])))
    T = int(r.integers(200, 3000))
    d = int(r.choice([64, 128, 192, 200, 256, 320]))
    F = int(r.choice([64, 72, 128, 192, 256]))
    grid_cap = int(r.choice([-1, 2, 3, 5, 9]))
    rank = int(r.integers(-1, D))
    _say("whole path, random shape", dict(T=T, d=d, E=E, k=k, F=F, D=D, grid_cap=grid_cap, rank=rank))
    w = WL.small(T=T, d=d, E=E, k=k, F=F, D=D, dtype="bf16", C=max(1, min(4, E // max(1, E // D))))
    m = S.SemMoE(S.Config.from_workload(w), allocate_workspace=False)
    try:
        m.set_tuning(4, grid_cap)
        lay, inp, ids, want_w, dw, Y, Yo, weights = _run_path(w, rank=rank)
        H.assert_close(Y, Yo, "bf16", "Y")
        if rank < 0:
            out = lay.combine()
            H.assert_close(out, O.moe_definition(inp.X, ids, want_w, lambda e: weights[e]), "bf16", "Out")
    finally:
        m.set_tuning(4, -1)
