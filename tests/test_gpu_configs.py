"""GPU parity at the five full workload sizes, in the launch configuration the benchmark times.

Integer stages are compared in full, bit for bit.  Floating-point stages: logits in full; sampled X_perm
rows; the expert FFN of one rank - the launch the benchmark times, `expert_ffn(rank)` - on every row of that
rank, with the real weights of every expert on the device; the all-ranks launch on sampled rows of every
expert; and the layer output on at least 256 sampled tokens against the plain MoE definition.
"""
import math
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import workloads as WL
from oracle import semmoe_oracle as O
import paper_2503_04398_amd as S
from tests import harness as H

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1100)]


def _say(*a):
    print(*a, flush=True)


def _lp_optimum(g, D, cap):
    """max sum_i g[i, a_i] with at most `cap` tokens per rank, by scipy's LP solver"""
    from scipy.optimize import linprog
    from scipy.sparse import coo_matrix
    T = g.shape[0]
    cols = np.arange(T * D)
    one_rank = coo_matrix((np.ones(T * D), (np.repeat(np.arange(T), D), cols)), shape=(T, T * D)).tocsr()
    per_rank = coo_matrix((np.ones(T * D), (np.tile(np.arange(D), T), cols)), shape=(D, T * D)).tocsr()
    res = linprog(-g.astype(np.float64).ravel(), A_ub=per_rank, b_ub=np.full(D, cap), A_eq=one_rank, b_eq=np.ones(T),
                  bounds=(0, 1), method="highs")
    assert res.status == 0
    return int(round(-res.fun))


def _no_gainful_closed_walk(g, token_rank, D, cap):
    """Optimality certificate of an assignment at any size: its residual graph on the ranks (+ a node for free
    room) has no closed walk of positive gain.  Checked with a library routine: an arc of gain w gets the weight
    1 - (D + 2) * w (never zero, which scipy would drop); a simple closed walk of L <= D + 1 arcs and total gain G
    weighs L - (D + 2) * G, negative exactly when G >= 1, and scipy's Bellman-Ford reports negative cycles."""
    from scipy.sparse import csr_matrix
    from scipy.sparse.csgraph import bellman_ford, NegativeCycleError
    N, scale = D + 1, D + 2
    W = np.zeros((N, N))
    cnt = np.bincount(token_rank, minlength=D)
    for a in range(D):
        on = np.flatnonzero(token_rank == a)
        for b in range(D):
            if a != b and len(on):
                W[a, b] = -scale * int((g[on, b] - g[on, a]).max()) + 1
        if cnt[a] < cap:
            W[a, D] = 1
        W[D, a] = 1
    try:
        bellman_ford(csr_matrix(W), directed=True)
    except NegativeCycleError:
        return False
    return True


def _max_row_err(got, want):
    """largest over the rows of max|a-b| over the row / max|b| over the row: the tolerance measure applied row by
    row, so that rows of small magnitude are not judged against the largest element of the whole tensor"""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.abs(want).max(axis=1)
    num = np.abs(got - want).max(axis=1)
    return float((num / np.where(den > 0, den, 1.0)).max()) if len(den) else 0.0


def _full_config(name, n_tok_sample, n_slot_sample, rank):
    w = WL.CONFIGS[name]
    t0 = time.time()
    inp = H.make_inputs(w)
    lay = H.Layer(w)
    # ---- route
    logits, ids, tw = lay.route(inp)
    want_logits = O.route_logits(inp.X, inp.W_r, None, inp.token_class, inp.class_bias)
    err = O.max_rel_err(logits, want_logits)
    _say("  [%5.1fs] logits err %.2e" % (time.time() - t0, err))
    assert err <= 1e-5
    want_ids, want_w = H.oracle_select(w, logits)
    assert (ids == want_ids).all()
    assert O.max_rel_err(tw, want_w) <= 1e-5
    flips = (want_ids != H.oracle_select(w, want_logits)[0]).any(axis=1).mean()
    _say("  [%5.1fs] ids bit-exact on the GPU's logits; tokens whose ids differ under oracle logits: %.4f"
         % (time.time() - t0, flips))
    # ---- offline: profile batch -> histogram -> placement
    pinp = H.make_inputs(w, profile=True)
    play = H.Layer(w, T=pinp.X.shape[0])
    plog, pids, _ = play.route(pinp)
    assert (pids == H.oracle_select(w, plog)[0]).all()
    load, co, (e2r, phys, inv) = play.profile_placement(play.ids)
    ol, oc = O.coact_hist(pids, w.E)
    assert (load == ol).all() and (co == oc).all()
    oe2r, ophys, oinv = O.place(ol, oc, w.D)
    assert (e2r == oe2r).all() and (phys == ophys).all() and (inv == oinv).all()
    # the table-driven row: activation table of the profile batch by token key, then the schedule table
    V = WL.vocab_size(w)
    pkeys = WL.token_key(w, profile=True)
    table = H.to_np(play.token_expert_hist(pkeys, pids, V)).astype(np.int64)
    assert (table == O.token_expert_table(pkeys, pids, V, w.E)).all()
    sched = play.m.lookup_tables(table.astype(np.uint32), e2r)
    for g, x, nm in zip(sched, O.lookup_tables(table, e2r, w.D, w.k), ("dev", "conf_q16", "level")):
        assert (g == x).all(), nm
    # the inter-layer table: device sequences of two stand-in earlier layers (this layer's experts shifted by the
    # layer number, so the history is informative), activation table keyed by them, A / A_p from it
    VA = w.D * w.D
    pseq = None
    for layer in (2, 1):
        pseq = play.device_sequence((pids + layer) % w.E, e2r, pseq)
    table_a = H.to_np(play.token_expert_hist(pseq, pids, VA)).astype(np.int64)
    assert (table_a == O.token_expert_table(pseq, pids, VA, w.E)).all()
    sched_a = play.m.lookup_tables(table_a.astype(np.uint32), e2r)
    for g, x, nm in zip(sched_a, O.lookup_tables(table_a, e2r, w.D, w.k), ("dev_a", "conf_a_q16", "level_a")):
        assert (g == x).all(), nm
    del play, pinp
    _say("  [%5.1fs] coact_hist, place, token-expert table, sequence table and schedule tables bit-exact"
         % (time.time() - t0))
    # ---- reshuffle, dispatch
    lay.set_placement(e2r, phys, inv)
    got = lay.reshuffle()
    want = O.reshuffle(ids, e2r, w.D, w.cap)
    for g, x, nm in zip(got, want, ("token_rank", "shf", "inv_shf", "rank_count")):
        assert (g == x).all(), nm
    # the next row: gain-aware spill rounds at the full size (three rounds), bit for bit, and what they buy
    got3 = lay.reshuffle_rounds(3)
    want3 = O.reshuffle_rounds(ids, e2r, w.D, w.cap, 3)
    for g, x, nm in zip(got3, want3, ("token_rank", "shf", "inv_shf", "rank_count")):
        assert (g == x).all(), "rounds: " + nm
    _say("  [%5.1fs] reshuffle with 3 spill rounds bit-exact; remote-pair fraction %.4f (1 round: %.4f)"
         % (time.time() - t0, O.remote_fraction(ids, e2r, want3[0]), O.remote_fraction(ids, e2r, want[0])))
    # moves of placed tokens after the three rounds, until nothing is left to gain (one workgroup: up to 16 ranks)
    if w.D <= 16 and w.k <= 15 and w.T <= 32768:
        gotr, cycles, conv = lay.reshuffle_refine(3)
        wantr, wcycles, wconv = O.reshuffle_refine(ids, e2r, w.D, w.cap, rounds=3)
        assert (cycles, conv) == (wcycles, 1) and wconv
        for g, x, nm in zip(gotr, wantr, ("token_rank", "shf", "inv_shf", "rank_count")):
            assert (g == x).all(), "refine: " + nm
        # the optimum of the assignment problem from a library solver (the LP of a transportation problem is integral)
        g_all = O.gain_matrix(ids, e2r, w.D)
        assert _no_gainful_closed_walk(g_all, gotr[0], w.D, w.cap)
        assert not _no_gainful_closed_walk(g_all, got3[0], w.D, w.cap) or cycles == 0   # the certificate can fail
        lp = ""
        if w.T * w.D <= 70000:
            assert O.local_pairs(ids, e2r, gotr[0]) == _lp_optimum(g_all, w.D, w.cap)
            lp = " = LP optimum"
        _say("  [%5.1fs] reshuffle refined to the optimum in %d cycles, bit-exact; remote-pair fraction %.4f%s"
             % (time.time() - t0, cycles, O.remote_fraction(ids, e2r, gotr[0]), lp))
    # the table-driven row at the full size: rebatch from token keys alone, two thresholds
    keys = WL.token_key(w)
    for thr in (0, 24576):
        gotl = lay.reshuffle_lookup(keys, sched[0], sched[1], sched[2], thr)
        wantl = O.reshuffle_lookup(keys, sched[0], sched[1], sched[2], thr, w.D, w.cap)
        for g, x, nm in zip(gotl, wantl, ("token_rank", "shf", "inv_shf", "rank_count")):
            assert (g == x).all(), "lookup: " + nm
        _say("  [%5.1fs] reshuffle from the schedule table (thr %.3f) bit-exact; remote-pair fraction %.4f"
             % (time.time() - t0, thr / 65536, O.remote_fraction(ids, e2r, wantl[0])))
    # Alg. 3 with both tables at the full size; 30 % of the keys are shared by all classes and lie outside T
    seq, wseq = None, None
    for layer in (2, 1):
        seq = lay.device_sequence((ids + layer) % w.E, e2r, seq)
        wseq = O.device_sequence((ids + layer) % w.E, e2r, w.D, wseq)
    assert (seq == wseq).all()
    skeys = WL.token_key(w, shared_frac=0.3)
    gotc = lay.reshuffle_cond(skeys, sched, seq, sched_a, 0)
    wantc = O.reshuffle_cond(skeys, *sched, seq, *sched_a, 0, w.D, w.cap)
    for g, x, nm in zip(gotc, wantc, ("token_rank", "shf", "inv_shf", "rank_count")):
        assert (g == x).all(), "cond: " + nm
    _say("  [%5.1fs] device sequences and reshuffle from both tables bit-exact; remote-pair fraction %.4f"
         % (time.time() - t0, O.remote_fraction(ids, e2r, wantc[0])))
    # the request-level row at the full size: requests = runs of tokens of one topic, ranks from the schedule table
    roff, _, rkeys = WL.requests(w)
    gotq = lay.request_schedule(roff, rkeys, sched[0])
    wrr = O.request_schedule(roff, rkeys, sched[0], w.D)
    for g, x, nm in zip(gotq, (wrr,) + O.request_assignment(roff, wrr, w.D),
                        ("req_rank", "token_rank", "shf", "inv_shf", "rank_count")):
        assert (g == x).all(), "request schedule: " + nm
    _say("  [%5.1fs] request schedule of %d requests bit-exact" % (time.time() - t0, len(roff) - 1))
    got = lay.reshuffle()          # the layer below runs on the plain reshuffle
    tr, shf, ishf, rc = want
    dg = lay.dispatch()
    dw = O.dispatch(None, ids, tr, ishf, phys, w.D)
    for nm in ("slot_of_pair", "pair_of_slot", "expert_offsets", "rank_offsets", "send_matrix"):
        assert (dg[nm] == dw[nm]).all(), nm
    assert int(dg["remote_pairs"]) == int(dw["remote_pairs"])
    P = w.P
    rs = np.random.default_rng(7)
    slots = np.sort(rs.choice(P, min(4096, P), replace=False))
    xp = H.to_np(lay.X_perm[torch.from_numpy(slots).to(H.DEV)])
    assert (xp == inp.X[dw["pair_of_slot"][slots] // w.k]).all()
    v_e2r, _, _ = O.vanilla_placement(w.E, w.D)
    home = O.home_rank(w.T, w.D)
    _say("  [%5.1fs] reshuffle/dispatch bit-exact; remote-pair fraction vanilla %.4f, placed %.4f, placed+reshuffle %.4f"
         % (time.time() - t0, O.remote_fraction(ids, v_e2r, home), O.remote_fraction(ids, e2r, home),
            int(dw["remote_pairs"]) / P))
    # ---- FFN + combine.  Every expert's real weights are drawn (a thread pool ahead of the loop, a few experts in
    # flight so that host memory stays flat), uploaded, and the oracle's share for that expert is computed while they
    # are at hand: every row of `rank` (the launch the benchmark times), sampled slots of every expert (the all-ranks
    # launch) and that expert's term of the plain MoE definition on the sampled tokens.
    toks = np.sort(rs.choice(w.T, min(n_tok_sample, w.T), replace=False))
    pos = dw["pair_of_slot"]
    off = dw["expert_offsets"].astype(np.int64)
    r_lo, r_hi = int(dw["rank_offsets"][rank]), int(dw["rank_offsets"][rank + 1])
    samp = np.sort(rs.choice(P, min(n_slot_sample, P), replace=False))
    Yo_rank = np.zeros((r_hi - r_lo, w.d), dtype=np.float64)
    Yo_samp = np.zeros((len(samp), w.d), dtype=np.float64)
    lay.W_gu = torch.empty(w.E, 2 * w.F, w.d, dtype=H.act_dtype(w), device=H.DEV)
    lay.W_down = torch.empty(w.E, w.d, w.F, dtype=H.act_dtype(w), device=H.DEV)
    lay._loaded = set(range(w.E))
    pool = ThreadPoolExecutor(max_workers=8)
    ahead = 12
    futs = {e: pool.submit(WL.expert_weight, w, e) for e in range(min(ahead, w.E))}
    seen = []

    def weight_of(e):
        """weights of expert e, drawn once; uploads them and computes the oracle rows that need them"""
        assert e not in seen
        seen.append(e)
        wgu, wdn = futs.pop(e).result()
        nxt = max(list(futs) + [e]) + 1
        if nxt < w.E:
            futs[nxt] = pool.submit(WL.expert_weight, w, nxt)
        lay.W_gu[e].copy_(H.to_dev(wgu, w))
        lay.W_down[e].copy_(H.to_dev(wdn, w))
        wgu, wdn = wgu.astype(np.float64), wdn.astype(np.float64)   # once: the oracle's FFN works in fp64
        q = int(phys[e])
        lo, hi = int(off[q]), int(off[q + 1])
        if e2r[e] == rank and hi > lo:
            Yo_rank[lo - r_lo:hi - r_lo] = O.swiglu_ffn(inp.X[pos[lo:hi] // w.k], wgu, wdn)
        a, b = np.searchsorted(samp, [lo, hi])
        if b > a:
            Yo_samp[a:b] = O.swiglu_ffn(inp.X[pos[samp[a:b]] // w.k], wgu, wdn)
        if (e + 1) % 32 == 0:
            _say("  [%5.1fs] ... %d experts" % (time.time() - t0, e + 1))
        return wgu, wdn

    used = set(int(e) for e in np.unique(ids[toks]))
    todo = iter(range(w.E))

    def weight_in_order(e):
        """the definition asks for the experts its tokens use, in ascending id; the ones in between are done on the way"""
        for e2 in todo:
            r = weight_of(e2)
            if e2 == e:
                return r
        raise AssertionError("experts are asked for in ascending order")

    shared = WL.shared_weight(w) if w.n_shared else None
    ref = O.moe_definition_by_expert(inp.X, ids, want_w, weight_in_order, shared, tokens=toks)
    for e2 in todo:
        weight_of(e2)
    pool.shutdown()
    assert seen == list(range(w.E)) and used <= set(seen)
    _say("  [%5.1fs] all %d experts' weights drawn and uploaded; oracle rows computed (%d of rank %d, %d sampled, "
         "%d tokens)" % (time.time() - t0, w.E, r_hi - r_lo, rank, len(samp), len(toks)))
    # (1) the launch the benchmark times: the experts of `rank` alone; every row of the rank, the rest untouched
    Y = lay.expert_ffn(rank, poison=512.0)
    assert bool((Y[:r_lo] == 512.0).all()) and bool((Y[r_hi:] == 512.0).all())
    Y_rank = H.to_np(Y[r_lo:r_hi])
    e_all = H.assert_close(Y_rank, Yo_rank, w.dtype, "Y rows of rank %d" % rank)
    e_row = _max_row_err(Y_rank, Yo_rank)
    assert e_row <= H.TOL[w.dtype], "a row of rank %d is off by %.3e of its own largest element" % (rank, e_row)
    _say("  [%5.1fs] expert_ffn(%d): all %d rows within tolerance (tensor %.2e, worst row against its own maximum %.2e)"
         % (time.time() - t0, rank, r_hi - r_lo, e_all, e_row))
    # (2) all ranks in one launch
    Y2 = lay.expert_ffn(-1)
    H.assert_close(H.to_np(Y2[torch.from_numpy(samp).to(H.DEV)]), Yo_samp, w.dtype, "sampled Y rows, all ranks")
    same = bool((Y2[r_lo:r_hi] == Y[r_lo:r_hi]).all())
    ysh = None
    if w.n_shared:
        ysh = lay.shared_ffn()
        H.assert_close(H.to_np(ysh[torch.from_numpy(toks).to(H.DEV)]), O.swiglu_ffn(inp.X[toks], *shared), w.dtype,
                       "Y_shared")
    out = lay.combine(Y_shared=ysh)
    e2 = H.assert_close(out[toks], ref, w.dtype, "Out vs plain MoE definition")
    e2r_ = _max_row_err(out[toks], ref)
    assert e2r_ <= H.TOL[w.dtype]
    _say("  [%5.1fs] expert_ffn(-1): %d sampled rows within tolerance (rank %d's rows bitwise equal to its own launch: "
         "%s); layer output on %d tokens vs the plain MoE definition: %.2e (worst row %.2e)"
         % (time.time() - t0, len(samp), rank, same, len(toks), e2, e2r_))


@pytest.mark.parametrize("name,n_tok,n_slot,rank", [
    ("c1_tiny_fp32", 256, 512, 0),
    ("c2_qwen3_30b", 512, 4096, 0),
    ("c5_qwen3_235b_decode", 256, 2048, 0),
    ("c4_gpt_oss_120b", 256, 2048, 0),
    ("c3_deepseek_v3", 256, 1024, 0),
])
def test_full_config(name, n_tok, n_slot, rank):
    _say("full config", name)
    _full_config(name, n_tok, n_slot, rank)
