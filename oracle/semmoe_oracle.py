"""CPU oracle for the semantic-parallel MoE layer (Sem-MoE, arxiv 2503.04398).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow reference that the HIP
library is checked against.  Only the tests, the smoke check and the
`cpu_baseline` leg of the benchmark may import it; the product path never does.
It shares no code, tables or helpers with the HIP path.

Floating point is fp64 (inputs are taken as given, e.g. bf16-rounded values held
in float32) except where a decision must be taken in the kernel's precision:
the top-k selection works on fp32 logits, and the sigmoid score is an fp32
recipe fixed operation by operation (see `sigmoid_f32`).  Integers are int64.

Notation follows the paper: T tokens, d hidden, E experts (the paper's N),
k experts per token, D logical EP ranks (the paper's E / G / Q), m = E/D.
Pair index p = i*k + j (token i, slot j).

Which passage each function follows
  route_logits / select_topk   gating function G(h) = top-k(softmax(W_g h + b_g))  (Sec. 3.2)
  coact_hist                   token->expert activation counts (Sec. 3.2) in their
                               key-free form; expert-expert affinity of Alg. 1
  place                        Alg. 1 `expert_place` (+ App. B text), request term dropped
  reshuffle                    Alg. 3 `rebatch_tokens` (argsort, group, align, concat)
  reshuffle_rounds             the same with gain-aware spill rounds (towards the Sec. 3.3 optimum)
  reshuffle_refine             the same followed by moves of placed tokens until the Sec. 3.3 optimum is reached
  token_expert_table / lookup_tables / reshuffle_lookup
                               token-to-expert activation table and confidence (Sec. 3.2), the
                               schedule table T / T_p, and Alg. 3 `rebatch_tokens` driven by it
  device_sequence / reshuffle_cond
                               the inter-layer device-sequence table A / A_p (App. B) and Alg. 3's
                               cond(T_p > A_p, T, A) with both tables
  request_schedule / request_assignment
                               Alg. 2 `get_dp_rank` + `schedule` (Attention-DP scenario), with
                               S_r = argmax_j sum_{i in r} R_ij of Sec. 3.3
  expert_place_affinity / unit_schedule / coschedule_score / coschedule / token_labels
                               Alg. 1 whole (App. B): `expert_place` with its request term, `req_sched`,
                               the alternation and its score, the token labels T / T_p it ends with
  reshuffle_exact              the ILP's communication term (Sec. 3.3) solved exactly
                               for fixed placement: min-cost flow
  dispatch / combine           the two all2all of expert parallelism (Sec. 1) as
                               single-device permutations; `resume_tokens` of Alg. 3
  expert_ffn                   the expert FFN (Sec. 2), SwiGLU form
  moe_definition / moe_definition_by_expert
                               the plain MoE layer: what the whole path must equal
                               ("losslessly", Sec. 5), token by token / expert by expert
  remote volume                alpha*k*B*S/G all2all volume model (Sec. 3.1)

Pins (tests/test_oracle_*.py): brute force on tiny inputs, closed forms,
library argsort / matmul special cases, the 1/D local-activation rate of
class-free routing (the ~25 % baseline of Tables 3-4 at D = 4), planted-cluster
recovery; for the rows built on top: spill rounds - hand example, round one = the
greedy, greedy <= rounds <= optimum; moves of placed tokens - hand examples of an exchange, a rotation over
three ranks, a move into free room and of which walk and tokens are taken, the optimum of the
min-cost flow and of brute force, the budget of cycles; table-driven rebatch - counts, hand example,
threshold extremes, one key per token = the rebatch on the actual top-k; request
scheduling - hand example with mask and reset, the request-to-cluster rule where
the mask cannot bite, every round reaches every rank, brute force over the unmasked
set; co-scheduling solver - without the request term it is `place`, hand examples of every
term and of the swap gain, planted topics recovered, remote mass = remote pair count when
every token is a unit, never below the brute-force optimum, labels = `lookup_tables` of the
count table; device sequences and cond(T_p > A_p, T, A) - hand examples, the device is the first
arg-max of the gain matrix, one table missing = the rebatch from the other, per token the table
of higher confidence.  Parity unpinned (the paper gives nothing to check against): the
values of alpha, gamma, ft_steps; the behaviour of `align`; Fig. 3's example.
"""
from __future__ import annotations

import itertools
from typing import Dict, Optional, Tuple

import numpy as np

# --------------------------------------------------------------------------------------------
# a1  route
# --------------------------------------------------------------------------------------------


def route_logits(X, W_r, b_g=None, token_class=None, class_bias=None) -> np.ndarray:
    """logits[i,e] = sum_c X[i,c] W_r[e,c] + b_g[e] + class_bias[token_class[i], e], in fp64,
    rounded once to fp32 (gating function, Sec. 3.2; the class term is the synthetic
    context-independent token->expert affinity).  token_class = -1 adds nothing."""
    L = np.asarray(X, dtype=np.float64) @ np.asarray(W_r, dtype=np.float64).T
    if b_g is not None:
        L = L + np.asarray(b_g, dtype=np.float64)[None, :]
    if token_class is not None and class_bias is not None:
        tc = np.asarray(token_class)
        cb = np.asarray(class_bias, dtype=np.float64)
        has = tc >= 0
        L[has] += cb[tc[has]]
    return L.astype(np.float32)


# fp32 constants of the sigmoid recipe (each literal is rounded to fp32 once)
_LOG2E = np.float32(1.4426950408889634)
_EXP2_COEF = [np.float32(c) for c in (
    1.0,
    0.6931471805599453,      # ln2
    0.2402265069591007,      # ln2^2/2
    0.05550410866482158,     # ln2^3/6
    0.009618129107628477,    # ln2^4/24
    0.0013333558146428443,   # ln2^5/120
    0.00015403530393381608,  # ln2^6/720
)]


def sigmoid_f32(x: np.ndarray) -> np.ndarray:
    """Sigmoid as a fixed sequence of individually rounded fp32 operations (no fused
    multiply-add), so that a kernel executing the same sequence gets the same bits:
        x <- clamp(x, -30, 30);  t = (-x) * log2(e);  n = rint(t);  f = t - n
        p = c6;  p = p*f + c_i  for i = 5..0   (multiply, round, add, round)
        z = p * 2^n (exact);  s = 1 / (1 + z)  (correctly rounded add and divide)
    with c_i = ln(2)^i / i! rounded to fp32.  Accuracy: a few ulp."""
    x = np.asarray(x, dtype=np.float32)
    x = np.minimum(np.maximum(x, np.float32(-30.0)), np.float32(30.0))
    t = (-x) * _LOG2E
    n = np.rint(t)
    f = t - n
    p = np.full_like(f, _EXP2_COEF[6])
    for i in range(5, -1, -1):
        p = p * f
        p = p + _EXP2_COEF[i]
    z = np.ldexp(p, n.astype(np.int32)).astype(np.float32)
    s = np.float32(1.0) / (np.float32(1.0) + z)
    assert s.dtype == np.float32
    return s


def _topk_desc_lowidx(v: np.ndarray, k: int) -> np.ndarray:
    """indices of the k largest entries of a 1-D array, descending value, ties -> lower index"""
    order = sorted(range(len(v)), key=lambda e: (-v[e], e))
    return np.array(order[:k], dtype=np.int64)


def select_topk(logits, k: int, score: str = "softmax", renorm: bool = False, n_group: int = 1,
                topk_group: int = 1, routed_scale: float = 1.0, sel_bias=None):
    """Top-k expert ids and combine weights from fp32 logits (gating function, Sec. 3.2).

    softmax: choose the k largest logits (softmax is monotone), descending, ties -> lower
      expert id; weight = softmax over all E experts (fp64, max-subtracted) at the chosen ids,
      divided by their sum when `renorm`.
    sigmoid (group-limited, the DeepSeek-V3-style router named by the workload, not by the
      paper): s = sigmoid_f32(logit); s' = s + sel_bias (fp32); experts form n_group contiguous
      groups; group score = sum (fp32) of the group's two largest s'; keep the topk_group best
      groups (ties -> lower group); choose the k largest s' among their experts; weight =
      s[id] / sum_j s[id_j] * routed_scale (fp64) when `renorm`, else s[id] * routed_scale.
    Returns (ids[T,k] int32, w[T,k] float64)."""
    L = np.asarray(logits)
    assert L.dtype == np.float32, "selection is defined on fp32 logits"
    assert np.isfinite(L).all()
    T, E = L.shape
    assert 1 <= k <= E
    ids = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k), dtype=np.float64)
    if score == "softmax":
        for i in range(T):
            sel = _topk_desc_lowidx(L[i], k)
            z = L[i].astype(np.float64)
            z = np.exp(z - z.max())
            p = z / z.sum()
            wi = p[sel]
            if renorm:
                wi = wi / wi.sum()
            ids[i], w[i] = sel, wi
        return ids, w
    assert score == "sigmoid"
    assert E % n_group == 0 and 1 <= topk_group <= n_group
    gs = E // n_group
    assert k <= topk_group * gs
    s = sigmoid_f32(L)
    sb = np.zeros(E, dtype=np.float32) if sel_bias is None else np.asarray(sel_bias, dtype=np.float32)
    sp = s + sb[None, :]
    assert sp.dtype == np.float32
    for i in range(T):
        if n_group > 1:
            gscore = np.zeros(n_group, dtype=np.float32)
            for g in range(n_group):
                seg = sp[i, g * gs:(g + 1) * gs]
                if gs >= 2:
                    top2 = _topk_desc_lowidx(seg, 2)
                    gscore[g] = np.float32(seg[top2[0]]) + np.float32(seg[top2[1]])
                else:
                    gscore[g] = seg[0]
            keep = _topk_desc_lowidx(gscore, topk_group)
            allowed = np.zeros(E, dtype=bool)
            for g in keep:
                allowed[g * gs:(g + 1) * gs] = True
        else:
            allowed = np.ones(E, dtype=bool)
        cand = [e for e in range(E) if allowed[e]]
        cand.sort(key=lambda e: (-sp[i, e], e))
        sel = np.array(cand[:k], dtype=np.int64)
        wi = s[i, sel].astype(np.float64)
        if renorm:
            wi = wi / wi.sum()
        ids[i], w[i] = sel, wi * float(routed_scale)
    return ids, w


# --------------------------------------------------------------------------------------------
# a2  coact_hist
# --------------------------------------------------------------------------------------------


def coact_hist(ids, E: int, load=None, coact=None):
    """load[e] = #{(i,j): ids[i,j] = e};  coact[a,b] = #{i: a in ids[i] and b in ids[i]} for all
    ordered (a,b), a = b included (activation counts of Sec. 3.2 summed over token ids; the
    expert-expert affinity Alg. 1 consumes).  Accumulates into `load`/`coact` when given."""
    ids = np.asarray(ids)
    load = np.zeros(E, dtype=np.int64) if load is None else load
    coact = np.zeros((E, E), dtype=np.int64) if coact is None else coact
    for row in ids:
        for a in row:
            load[a] += 1
            for b in row:
                coact[a, b] += 1
    return load, coact


# --------------------------------------------------------------------------------------------
# a3  place  (Alg. 1 expert_place)
# --------------------------------------------------------------------------------------------


def place(load, coact, D: int, alpha: int = 1, gamma: int = 0, ft_passes: int = 8):
    """Balanced expert -> rank placement (Alg. 1 `expert_place`, request-affinity term dropped
    because this path has no requests).

    Greedy pass: experts in order of load, hottest first (ties -> lower id).  For expert e and
    every rank c that is not full:  EAfE[e,c] = sum of coact[e,e'] over experts e' already on c;
    score = alpha*EAfE[e,c] - gamma*loads_cls[c].  e goes to the arg-max rank (ties -> smaller
    loads_cls, then smaller c); a rank holding E/D experts is masked.
    Fine-tuning: the algorithm's random pair swaps "kept if the affinity gain is positive" are
    taken as deterministic first-improvement sweeps over pairs e1 < e2 on different ranks, at
    most `ft_passes` sweeps, stopping after a sweep without a swap.  The gain of a swap weighs
    both terms of the Sec. 3.3 objective with the weights of the greedy pass:
        gain = alpha * (change of the intra-rank co-activation mass W = sum_c sum_{a<b on c} coact[a,b])
             + gamma * (max(L1, L2) - max(L1', L2')),
    L1, L2 the loads of the two ranks before and L1', L2' after the swap (what the swap takes off
    the larger of the two loads: the maximum load over all ranks never grows by a swap whose load
    term is not negative).  With gamma = 0 this is the affinity gain alone.
    Physical order: rank-major, ascending original id inside a rank.
    Returns (expert_to_rank[E], phys_of_expert[E], expert_of_phys[E]) int32."""
    load = np.asarray(load, dtype=np.int64)
    A = np.asarray(coact, dtype=np.int64)
    E = load.shape[0]
    assert A.shape == (E, E) and E % D == 0
    m = E // D
    order = sorted(range(E), key=lambda e: (-int(load[e]), e))
    rank_of = [-1] * E
    members = [[] for _ in range(D)]
    loads_cls = [0] * D
    for e in order:
        best = None
        for c in range(D):
            if len(members[c]) >= m:       # masked
                continue
            eafe = sum(int(A[e, e2]) for e2 in members[c])
            score = alpha * eafe - gamma * loads_cls[c]
            key = (-score, loads_cls[c], c)
            if best is None or key < best[0]:
                best = (key, c)
        c = best[1]
        rank_of[e] = c
        members[c].append(e)
        loads_cls[c] += int(load[e])

    def aff(e, c, excl):
        """A(e, S) with S = experts on rank c other than e and `excl`"""
        on_c = np.array(rank_of) == c
        on_c[e] = False
        on_c[excl] = False
        return int(A[e][on_c].sum())

    for _ in range(ft_passes):
        swapped = False
        for e1 in range(E):
            for e2 in range(e1 + 1, E):
                c1, c2 = rank_of[e1], rank_of[e2]
                if c1 == c2:
                    continue
                g_e = aff(e1, c2, e2) + aff(e2, c1, e1) - aff(e1, c1, e1) - aff(e2, c2, e2)
                l1 = loads_cls[c1] - int(load[e1]) + int(load[e2])
                l2 = loads_cls[c2] - int(load[e2]) + int(load[e1])
                g_l = max(loads_cls[c1], loads_cls[c2]) - max(l1, l2)
                if alpha * g_e + gamma * g_l > 0:
                    rank_of[e1], rank_of[e2] = c2, c1
                    loads_cls[c1], loads_cls[c2] = l1, l2
                    swapped = True
        if not swapped:
            break
    expert_to_rank = np.array(rank_of, dtype=np.int32)
    phys = np.zeros(E, dtype=np.int32)
    seen = [0] * D
    for e in range(E):
        c = rank_of[e]
        phys[e] = c * m + seen[c]
        seen[c] += 1
    inv = np.zeros(E, dtype=np.int32)
    inv[phys] = np.arange(E, dtype=np.int32)
    return expert_to_rank, phys, inv


def vanilla_placement(E: int, D: int):
    """the original placement: expert e on rank e div m (the comparison baseline of Sec. 4.6)"""
    m = E // D
    e = np.arange(E, dtype=np.int32)
    return (e // m).astype(np.int32), e.copy(), e.copy()


def intra_rank_mass(coact, expert_to_rank) -> int:
    """W = sum over ranks of sum_{a<b on the rank} coact[a,b]"""
    A = np.asarray(coact, dtype=np.int64)
    r = np.asarray(expert_to_rank)
    E = len(r)
    return int(sum(int(A[a, b]) for a in range(E) for b in range(a + 1, E) if r[a] == r[b]))


# --------------------------------------------------------------------------------------------
# a4  reshuffle  (Alg. 3 rebatch_tokens)
# --------------------------------------------------------------------------------------------


def home_rank(T: int, D: int) -> np.ndarray:
    """the contiguous shard a plain reduce-scatter gives token i: i div ceil(T/D)"""
    per = -(-T // D)
    return (np.arange(T) // per).astype(np.int32)


def gain_matrix(ids, expert_to_rank, D: int) -> np.ndarray:
    """g[i,r] = #{j: expert_to_rank[ids[i,j]] = r}"""
    ids = np.asarray(ids)
    T, k = ids.shape
    g = np.zeros((T, D), dtype=np.int64)
    for i in range(T):
        for j in range(k):
            g[i, expert_to_rank[ids[i, j]]] += 1
    return g


def reshuffle(ids, expert_to_rank, D: int, cap: int):
    """Capacity-bounded token -> rank assignment and the shuffle permutation
    (Alg. 3 `rebatch_tokens`: device ids, argsort, group_by_key, align, concat).

    The per-token device id comes from the token's actual top-k against the placement (the
    perfect-predictor limit of the paper's lookup tables).  `align` is read as the capacity
    bound that makes all shards equal: at most `cap` tokens per rank, cap*D >= T.
      1. g[i,r]; pref(i) = argmax_r g[i,r], ties -> home(i) if it is a maximiser, else the
         smallest maximiser; conf(i) = g[i,pref(i)].
      2. keep: per rank the candidates {i: pref(i) = r} ordered by (conf desc, i asc); the first
         min(n_r, cap) stay on r.
      3. spill: the s-th spilled token (ascending i) takes the s-th free slot, free slots
         enumerated rank by rank in ascending rank order.
      4. shf = token indices stably sorted by token_rank (new position -> token);
         inv_shf[shf[q]] = q (`resume_tokens`).
    Returns (token_rank[T], shf[T], inv_shf[T], rank_count[D]) int32."""
    ids = np.asarray(ids)
    T, k = ids.shape
    assert cap * D >= T
    g = gain_matrix(ids, expert_to_rank, D)
    home = home_rank(T, D)
    pref = np.zeros(T, dtype=np.int64)
    conf = np.zeros(T, dtype=np.int64)
    for i in range(T):
        mx = g[i].max()
        if g[i, home[i]] == mx:
            pref[i] = home[i]
        else:
            pref[i] = int(np.flatnonzero(g[i] == mx)[0])
        conf[i] = mx
    token_rank = np.full(T, -1, dtype=np.int64)
    kept = np.zeros(D, dtype=np.int64)
    for r in range(D):
        cand = [i for i in range(T) if pref[i] == r]
        cand.sort(key=lambda i: (-conf[i], i))
        for i in cand[:cap]:
            token_rank[i] = r
        kept[r] = min(len(cand), cap)
    free_slots = [r for r in range(D) for _ in range(int(cap - kept[r]))]
    spilled = [i for i in range(T) if token_rank[i] < 0]
    for s, i in enumerate(spilled):
        token_rank[i] = free_slots[s]
    shf = np.argsort(token_rank, kind="stable")
    inv_shf = np.zeros(T, dtype=np.int64)
    inv_shf[shf] = np.arange(T)
    rank_count = np.bincount(token_rank, minlength=D)
    return (token_rank.astype(np.int32), shf.astype(np.int32), inv_shf.astype(np.int32),
            rank_count.astype(np.int32))


def reshuffle_rounds(ids, expert_to_rank, D: int, cap: int, rounds: int):
    """Capacity-bounded assignment with gain-aware spill rounds: the refinement of step 3 of
    `reshuffle` for the case where capacity binds (the objective of Sec. 3.3 for a fixed
    placement asks for the assignment with the most local pairs; `align` of Alg. 3 only asks for
    equal shards).  Instead of sending every spilled token to whatever slot is free, the tokens
    that are still unplaced propose again, each to its best rank among those that still have room:
      round t = 0 .. rounds-1:  room = ranks with a free slot;  every unplaced token i proposes
        pref_t(i) = argmax over ranks with room of g[i,r] (ties -> home(i) if it is such a
        maximiser, else the smallest), conf_t(i) = g[i, pref_t(i)];  rank r accepts its proposers
        in the order (conf desc, i asc) up to its free slots.
      then the tokens still unplaced take the remaining free slots in ascending rank order
        (ascending i), as in `reshuffle`.
    Round 0 is the keep phase of `reshuffle`, so rounds = 1 gives the same assignment.  Every
    round either fills a rank or places every proposer, so D rounds place everything that can
    be placed by proposal.  Returns (token_rank, shf, inv_shf, rank_count) int32."""
    ids = np.asarray(ids)
    T, k = ids.shape
    assert cap * D >= T and rounds >= 1
    g = gain_matrix(ids, expert_to_rank, D)
    home = home_rank(T, D)
    token_rank = np.full(T, -1, dtype=np.int64)
    free = np.full(D, cap, dtype=np.int64)
    for _ in range(rounds):
        room = [r for r in range(D) if free[r] > 0]
        proposers = {r: [] for r in room}
        for i in range(T):
            if token_rank[i] >= 0:
                continue
            mx = max(g[i, r] for r in room)
            if home[i] in proposers and g[i, home[i]] == mx:
                p = int(home[i])
            else:
                p = min(r for r in room if g[i, r] == mx)
            proposers[p].append((-int(mx), i))
        if not any(proposers.values()):
            break
        for r in room:
            proposers[r].sort()
            for _, i in proposers[r][:free[r]]:
                token_rank[i] = r
            free[r] -= min(free[r], len(proposers[r]))
    free_slots = [r for r in range(D) for _ in range(int(free[r]))]
    for s, i in enumerate([i for i in range(T) if token_rank[i] < 0]):
        token_rank[i] = free_slots[s]
    shf = np.argsort(token_rank, kind="stable")
    inv_shf = np.zeros(T, dtype=np.int64)
    inv_shf[shf] = np.arange(T)
    rank_count = np.bincount(token_rank, minlength=D)
    return (token_rank.astype(np.int32), shf.astype(np.int32), inv_shf.astype(np.int32),
            rank_count.astype(np.int32))


def reshuffle_refine(ids, expert_to_rank, D: int, cap: int, max_cycles: int = 1 << 30, rounds: int = 1, start=None):
    """`reshuffle_rounds` (rounds = 1: `reshuffle`), then moves of already placed tokens until no
    assignment under the capacity bound has more local pairs (the communication term of the
    Sec. 3.3 objective for a fixed placement; `align` of Alg. 3 as the bound).  An assignment is
    optimal exactly when its residual graph has no closed walk of positive gain, so such walks
    are cancelled one by one.  `start`, if given, is the assignment to begin with instead.

    Nodes: the D ranks and a node Z that stands for free room.  Arcs, for the current assignment:
      a -> b (ranks, a != b)  w = max over the tokens i on a of g[i,b] - g[i,a]  (absent if a is empty)
      a -> Z                  w = 0, present when a holds fewer than cap tokens
      Z -> b                  w = 0
    best_1 = w;  best_L[u][v] = max_x best_{L-1}[u][x] + w[x][v]  (walks of exactly L arcs).
    One cycle: take the smallest L in 2 .. D+1 for which some best_L[u][u] > 0 (a closed walk
    of that least length visits no node twice); u0 = the smallest u with the largest
    best_L[u][u]; walk back from u0, at every step to the smallest x with
    best_{l-1}[u0][x] + w[x][v] = best_l[u0][v].  n(a -> b) = number of tokens on a that attain
    w[a][b]; n(a -> Z) = cap - tokens on a; m = the least n over the arcs of the walk that leave
    a rank.  On every arc a -> b between ranks the m tokens of smallest index among those that
    attain w[a][b] move to b.  Every cycle adds at least m >= 1 local pairs, so the loop ends.

    Stops when no such walk is left (converged) or after `max_cycles` cycles.  Returns
    (token_rank, shf, inv_shf, rank_count) int32, cycles applied, converged (bool)."""
    ids = np.asarray(ids)
    T = ids.shape[0]
    assert cap * D >= T and max_cycles >= 0
    if start is None:
        token_rank = reshuffle_rounds(ids, expert_to_rank, D, cap, rounds)[0].astype(np.int64)
    else:
        token_rank = np.array(start, dtype=np.int64)
        assert token_rank.shape == (T,) and np.bincount(token_rank, minlength=D).max() <= cap
    g = gain_matrix(ids, expert_to_rank, D)
    N, Z = D + 1, D
    cycles, converged = 0, False
    while True:
        on = [np.flatnonzero(token_rank == a) for a in range(D)]
        w = [[None] * N for _ in range(N)]
        for a in range(D):
            for b in range(D):
                if a != b and len(on[a]) > 0:
                    w[a][b] = int((g[on[a], b] - g[on[a], a]).max())
            if len(on[a]) < cap:
                w[a][Z] = 0
            w[Z][a] = 0
        best = {1: w}
        found, u0 = None, None
        for L in range(2, N + 1):
            cur = [[None] * N for _ in range(N)]
            for u in range(N):
                for v in range(N):
                    sums = [best[L - 1][u][x] + w[x][v] for x in range(N)
                            if best[L - 1][u][x] is not None and w[x][v] is not None]
                    if sums:
                        cur[u][v] = max(sums)
            best[L] = cur
            diag = [cur[u][u] for u in range(N)]
            have = [d for d in diag if d is not None]
            if have and max(have) > 0:
                found, u0 = L, diag.index(max(have))
                break
        if found is None:
            converged = True
            break
        if cycles == max_cycles:
            break
        walk, v = [u0], u0
        for l in range(found, 1, -1):
            x = min(x for x in range(N)
                    if best[l - 1][u0][x] is not None and w[x][v] is not None
                    and best[l - 1][u0][x] + w[x][v] == best[l][u0][v])
            walk.append(x)
            v = x
        walk.append(u0)
        walk.reverse()
        movers, m = [], None
        for a, b in zip(walk[:-1], walk[1:]):
            if a == Z:
                continue
            if b == Z:
                n = cap - len(on[a])
            else:
                sel = on[a][(g[on[a], b] - g[on[a], a]) == w[a][b]]
                movers.append((b, sel))
                n = len(sel)
            m = n if m is None else min(m, n)
        for b, sel in movers:
            token_rank[sel[:m]] = b
        cycles += 1
    shf = np.argsort(token_rank, kind="stable")
    inv_shf = np.zeros(T, dtype=np.int64)
    inv_shf[shf] = np.arange(T)
    rank_count = np.bincount(token_rank, minlength=D)
    return (token_rank.astype(np.int32), shf.astype(np.int32), inv_shf.astype(np.int32),
            rank_count.astype(np.int32)), cycles, converged


# --------------------------------------------------------------------------------------------
# table-driven (predictive) reshuffle: the paper's online mechanism, from token ids alone
# --------------------------------------------------------------------------------------------


def token_expert_table(keys, ids, V: int, E: int, table=None) -> np.ndarray:
    """Token-to-expert activation table of Sec. 3.2: table[v,e] = #{(i,j): keys[i] = v and ids[i,j] = e},
    accumulated over profiling batches when `table` is passed back in."""
    keys = np.asarray(keys)
    ids = np.asarray(ids)
    if table is None:
        table = np.zeros((V, E), dtype=np.int64)
    for i in range(ids.shape[0]):
        for j in range(ids.shape[1]):
            table[keys[i], ids[i, j]] += 1
    return table


def lookup_tables(table, expert_to_rank, D: int, k: int):
    """Token-to-device schedule table and its confidence (the tables T and T_p of Alg. 2 / Alg. 3) from the
    activation table and a placement.  The confidence table of Sec. 3.2 is C_p[v,e] = table[v,e] / sum_e table[v,e];
    the probability that an activation of token v lands on device r is the sum of C_p over r's experts:
        mass[v,r] = sum_{e on r} table[v,e];   dev[v]  = argmax_r mass[v,r] (equal -> smallest r);
        T_p[v] = mass[v,dev[v]] / sum_r mass[v,r].
    Kept in integers so that every implementation takes the same decisions:
        conf_q16[v] = floor(65536 * T_p[v]);   level[v] = round-half-up(k * T_p[v]) in [0,k]
    (k * T_p is the number of the token's k activations expected on that device: the keep priority).
    A key never seen in profiling has dev = -1, conf_q16 = 0, level = 0.
    Returns (dev[V], conf_q16[V], level[V]) int32."""
    table = np.asarray(table, dtype=np.int64)
    V, E = table.shape
    e2r = np.asarray(expert_to_rank)
    dev = np.full(V, -1, dtype=np.int32)
    conf = np.zeros(V, dtype=np.int32)
    level = np.zeros(V, dtype=np.int32)
    for v in range(V):
        mass = [0] * D
        for e in range(E):
            mass[int(e2r[e])] += int(table[v, e])
        tot = sum(mass)
        if tot == 0:
            continue
        best = max(range(D), key=lambda r: (mass[r], -r))
        dev[v] = best
        conf[v] = (65536 * mass[best]) // tot
        level[v] = (2 * k * mass[best] + tot) // (2 * tot)
    return dev, conf, level


def reshuffle_lookup(keys, dev, conf_q16, level, thr_q16: int, D: int, cap: int):
    """`rebatch_tokens` of Alg. 3 as the paper runs it, before the gate: the device id of a token comes from
    the schedule table, dev_ids = cond(T_p[B] > A_p[B], T[B], A[B]).  The inter-layer table A is not built on
    this path: its device is read as the token's home shard and its confidence A_p as the constant thr_q16
    (in 1/65536).  So pref(i) = dev[keys[i]] and conf(i) = level[keys[i]] when conf_q16[keys[i]] > thr_q16
    (and the key was seen), else pref(i) = home(i), conf(i) = 0; then keep / spill / shuffle exactly as in
    `reshuffle` (steps 2-4).  Returns (token_rank, shf, inv_shf, rank_count) int32."""
    keys = np.asarray(keys)
    T = keys.shape[0]
    assert cap * D >= T
    home = home_rank(T, D)
    pref = np.zeros(T, dtype=np.int64)
    conf = np.zeros(T, dtype=np.int64)
    for i in range(T):
        v = int(keys[i])
        if dev[v] >= 0 and conf_q16[v] > thr_q16:
            pref[i], conf[i] = dev[v], level[v]
        else:
            pref[i], conf[i] = home[i], 0
    token_rank = np.full(T, -1, dtype=np.int64)
    kept = np.zeros(D, dtype=np.int64)
    for r in range(D):
        cand = [i for i in range(T) if pref[i] == r]
        cand.sort(key=lambda i: (-conf[i], i))
        for i in cand[:cap]:
            token_rank[i] = r
        kept[r] = min(len(cand), cap)
    free_slots = [r for r in range(D) for _ in range(int(cap - kept[r]))]
    for s, i in enumerate([i for i in range(T) if token_rank[i] < 0]):
        token_rank[i] = free_slots[s]
    shf = np.argsort(token_rank, kind="stable")
    inv_shf = np.zeros(T, dtype=np.int64)
    inv_shf[shf] = np.arange(T)
    return (token_rank.astype(np.int32), shf.astype(np.int32), inv_shf.astype(np.int32),
            np.bincount(token_rank, minlength=D).astype(np.int32))


def device_sequence(ids, expert_to_rank, D: int, seq_in=None) -> np.ndarray:
    """The device a token selects at a layer, appended to the sequence of the layers before (App. B, inter-layer
    activation conjugacy: the rows of the sequence table are the devices selected at the previous l layers).  With
    k experts per token the device selected is read as the one holding most of the token's k experts (equal ->
    the smallest).  seq_out[i] = seq_in[i]*D + device(i): chaining the call over l layers numbers the D^l rows,
    oldest layer most significant.  A token whose history is unknown (seq_in[i] < 0) stays unknown (-1).
    The sequence table itself is `token_expert_table` keyed by these numbers, and A / A_p are its `lookup_tables`."""
    ids = np.asarray(ids)
    e2r = np.asarray(expert_to_rank)
    T = ids.shape[0]
    out = np.zeros(T, dtype=np.int32)
    for i in range(T):
        cnt = [0] * D
        for e in ids[i]:
            cnt[int(e2r[int(e)])] += 1
        dev = max(range(D), key=lambda r: (cnt[r], -r))
        prev = 0 if seq_in is None else int(seq_in[i])
        out[i] = -1 if prev < 0 else prev * D + dev
    return out


def _rebatch_from_preferences(pref, conf, D: int, cap: int):
    """steps 2-4 of `reshuffle` for given preferences: keep by (conf desc, i asc) up to cap, spill the rest into the
    free slots in rank order, shuffle = stable argsort of the final ranks"""
    T = len(pref)
    token_rank = np.full(T, -1, dtype=np.int64)
    kept = [0] * D
    for r in range(D):
        cand = sorted((i for i in range(T) if pref[i] == r), key=lambda i: (-conf[i], i))
        for i in cand[:cap]:
            token_rank[i] = r
        kept[r] = min(len(cand), cap)
    free_slots = [r for r in range(D) for _ in range(cap - kept[r])]
    for s_, i in enumerate([i for i in range(T) if token_rank[i] < 0]):
        token_rank[i] = free_slots[s_]
    shf = np.argsort(token_rank, kind="stable")
    inv_shf = np.zeros(T, dtype=np.int64)
    inv_shf[shf] = np.arange(T)
    return (token_rank.astype(np.int32), shf.astype(np.int32), inv_shf.astype(np.int32),
            np.bincount(token_rank, minlength=D).astype(np.int32))


def reshuffle_cond(keys, dev, conf_q16, level, seq_keys, dev_a, conf_a_q16, level_a, thr_q16: int, D: int, cap: int):
    """`rebatch_tokens` of Alg. 3 with both of its tables: dev_ids = cond(T_p[B] > A_p[B], T[B], A[B]).  T is
    indexed by the token's key, the inter-layer table A by the token's device sequence (`device_sequence`); an
    entry that does not exist (index outside the table, or never profiled: dev < 0) has confidence -1, so the
    other table wins and, when neither exists, the token stays home.  The chosen entry is followed when its
    confidence exceeds thr_q16 (-1: always): pref = its device, conf = its level; otherwise pref = home, conf = 0.
    Then keep / spill / shuffle as in `reshuffle`.  Returns (token_rank, shf, inv_shf, rank_count) int32."""
    keys = np.asarray(keys)
    seq_keys = np.asarray(seq_keys)
    T = keys.shape[0]
    assert cap * D >= T
    home = home_rank(T, D)
    pref = [0] * T
    conf = [0] * T

    def entry(v, dv, cf, lv):
        v = int(v)
        if 0 <= v < len(dv) and 0 <= int(dv[v]) < D:
            return int(cf[v]), int(dv[v]), int(lv[v])
        return -1, -1, 0

    for i in range(T):
        ct, dt, lt = entry(keys[i], dev, conf_q16, level)
        ca, da, la = entry(seq_keys[i], dev_a, conf_a_q16, level_a)
        c, d_, l_ = (ct, dt, lt) if ct > ca else (ca, da, la)
        if c >= 0 and c > thr_q16:
            pref[i], conf[i] = d_, l_
        else:
            pref[i], conf[i] = int(home[i]), 0
    return _rebatch_from_preferences(pref, conf, D, cap)


def request_schedule(req_offsets, keys, dev, D: int) -> np.ndarray:
    """Online request scheduling of the Attention-DP scenario (Alg. 2 `get_dp_rank`, with the request-to-cluster
    rule S_r = argmax_j sum_{i in r} R_ij of Sec. 3.3).  The schedule table holds one device per token id, so its
    row read as a vector over devices is one-hot and the score of a request is a count:
        dev_score[r] = #{tokens i of the request: dev[keys[i]] = r}   (keys never profiled count nowhere).
    Requests are taken in arrival order; a request goes to the unmasked device of the highest score (equal ->
    the smallest id), that device is masked, and once every device is masked the mask is cleared: any D
    consecutive requests of a round land on D different devices.  Returns req_rank[n_req] int32."""
    off = np.asarray(req_offsets)
    keys = np.asarray(keys)
    n_req = off.shape[0] - 1
    req_rank = np.zeros(n_req, dtype=np.int32)
    dev_mask = [True] * D
    for q in range(n_req):
        dev_score = [0] * D
        for i in range(int(off[q]), int(off[q + 1])):
            r = int(dev[int(keys[i])])
            if r >= 0:
                dev_score[r] += 1
        best = -1
        for r in range(D):
            if dev_mask[r] and (best < 0 or dev_score[r] > dev_score[best]):
                best = r
        req_rank[q] = best
        dev_mask[best] = False
        if not any(dev_mask):
            dev_mask = [True] * D
    return req_rank


def request_assignment(req_offsets, req_rank, D: int):
    """`schedule(R, dev_id)` of Alg. 2 in the index form the rest of the path reads: every token inherits the rank
    of its request; shf = tokens stably sorted by rank (so a rank holds its requests in arrival order, each
    contiguous); inv_shf[shf[q]] = q.  No capacity bound: a DP rank holds whole requests.
    Returns (token_rank, shf, inv_shf, rank_count) int32."""
    off = np.asarray(req_offsets)
    T = int(off[-1])
    token_rank = np.zeros(T, dtype=np.int64)
    for q in range(off.shape[0] - 1):
        token_rank[int(off[q]):int(off[q + 1])] = int(req_rank[q])
    shf = np.argsort(token_rank, kind="stable")
    inv_shf = np.zeros(T, dtype=np.int64)
    inv_shf[shf] = np.arange(T)
    return (token_rank.astype(np.int32), shf.astype(np.int32), inv_shf.astype(np.int32),
            np.bincount(token_rank, minlength=D).astype(np.int32))


# --------------------------------------------------------------------------------------------
# the co-scheduling solver in full (Alg. 1 with its request half; App. B)
# --------------------------------------------------------------------------------------------


def expert_place_affinity(load, coact, D: int, unit_act=None, unit_rank=None, alpha_e: int = 1, beta_e: int = 0,
                          gamma_e: int = 0, ft_passes: int = 8):
    """`expert_place` of Alg. 1 with its request term.  A unit is a request (or a token key standing for all its
    occurrences); unit_act[u,e] is the activation mass of unit u on expert e, unit_rank[u] the cluster the unit is
    scheduled to at the moment (fixed during the call).
        EAfE[e,c] = sum of coact[e,e'] over experts e' already on c
        EAfR[e,c] = sum of unit_act[u,e] over units u scheduled to c
        score     = alpha_e*EAfE[e,c] + beta_e*EAfR[e,c] - gamma_e*loads_cls[c]
    Experts hottest first (equal -> lower id); arg-max over the clusters not yet full (equal -> smaller loads_cls,
    then smaller c); a cluster is full at E/D experts.  Fine-tuning as in `place`: first-improvement sweeps over
    pairs e1 < e2 on different clusters, gain = alpha_e*(change of the intra-cluster co-activation mass)
    + beta_e*(change of the activation mass that is local, sum_e EAfR[e, cluster(e)])
    + gamma_e*(what the swap takes off the larger of the two clusters' loads); swap when gain > 0.
    With beta_e = 0 this is `place`.  Returns expert_to_rank[E] int32."""
    load = np.asarray(load, dtype=np.int64)
    A = np.asarray(coact, dtype=np.int64)
    E = load.shape[0]
    assert A.shape == (E, E) and E % D == 0
    m = E // D
    R = [[0] * D for _ in range(E)]                 # EAfR
    if unit_act is not None and unit_rank is not None:
        Q = np.asarray(unit_act, dtype=np.int64)
        for u in range(Q.shape[0]):
            c = int(unit_rank[u])
            for e in range(E):
                R[e][c] += int(Q[u, e])
    order = sorted(range(E), key=lambda e: (-int(load[e]), e))
    rank_of = [-1] * E
    members = [[] for _ in range(D)]
    loads_cls = [0] * D
    for e in order:
        best = None
        for c in range(D):
            if len(members[c]) >= m:
                continue
            eafe = sum(int(A[e, e2]) for e2 in members[c])
            score = alpha_e * eafe + beta_e * R[e][c] - gamma_e * loads_cls[c]
            key = (-score, loads_cls[c], c)
            if best is None or key < best[0]:
                best = (key, c)
        c = best[1]
        rank_of[e] = c
        members[c].append(e)
        loads_cls[c] += int(load[e])

    def aff(e, c, excl):
        return sum(int(A[e, x]) for x in range(E) if rank_of[x] == c and x != e and x != excl)

    for _ in range(ft_passes):
        swapped = False
        for e1 in range(E):
            for e2 in range(e1 + 1, E):
                c1, c2 = rank_of[e1], rank_of[e2]
                if c1 == c2:
                    continue
                g_e = aff(e1, c2, e2) + aff(e2, c1, e1) - aff(e1, c1, e1) - aff(e2, c2, e2)
                g_r = R[e1][c2] + R[e2][c1] - R[e1][c1] - R[e2][c2]
                l1 = loads_cls[c1] - int(load[e1]) + int(load[e2])
                l2 = loads_cls[c2] - int(load[e2]) + int(load[e1])
                g_l = max(loads_cls[c1], loads_cls[c2]) - max(l1, l2)
                if alpha_e * g_e + beta_e * g_r + gamma_e * g_l > 0:
                    rank_of[e1], rank_of[e2] = c2, c1
                    loads_cls[c1], loads_cls[c2] = l1, l2
                    swapped = True
        if not swapped:
            break
    return np.array(rank_of, dtype=np.int32)


def placement_order(expert_to_rank, D: int):
    """physical order of a placement: rank-major, ascending original id inside a rank.
    Returns (phys_of_expert, expert_of_phys) int32."""
    r = np.asarray(expert_to_rank)
    E = r.shape[0]
    m = E // D
    phys = np.zeros(E, dtype=np.int32)
    seen = [0] * D
    for e in range(E):
        phys[e] = int(r[e]) * m + seen[int(r[e])]
        seen[int(r[e])] += 1
    inv = np.zeros(E, dtype=np.int32)
    inv[phys] = np.arange(E, dtype=np.int32)
    return phys, inv


def unit_schedule(unit_act, unit_len, expert_to_rank, D: int, alpha_r: int = 0, beta_r: int = 1) -> np.ndarray:
    """`req_sched` of Alg. 1: units longest first (equal -> lower index); for unit u and every cluster c that is
    not full
        RAfR[u,c] = sum over units u' already on c of sum_e unit_act[u,e]*unit_act[u',e]   (request-request)
        RAfE[u,c] = sum of unit_act[u,e] over experts e placed on c                          (request-expert)
        score     = alpha_r*RAfR[u,c] + beta_r*RAfE[u,c]
    u goes to the arg-max (equal -> the cluster holding fewer tokens so far, then smaller c); a cluster is full
    at ceil(U/D) units.  Returns unit_rank[U] int32."""
    Q = np.asarray(unit_act, dtype=np.int64)
    U, E = Q.shape
    ln = [int(x) for x in np.asarray(unit_len)]
    e2r = [int(x) for x in np.asarray(expert_to_rank)]
    cap = -(-U // D)
    order = sorted(range(U), key=lambda u: (-ln[u], u))
    on = [[] for _ in range(D)]
    tokens_cls = [0] * D
    unit_rank = np.zeros(U, dtype=np.int32)
    for u in order:
        best = None
        for c in range(D):
            if len(on[c]) >= cap:
                continue
            rafr = sum(int(Q[u, e]) * int(Q[u2, e]) for u2 in on[c] for e in range(E))
            rafe = sum(int(Q[u, e]) for e in range(E) if e2r[e] == c)
            score = alpha_r * rafr + beta_r * rafe
            key = (-score, tokens_cls[c], c)
            if best is None or key < best[0]:
                best = (key, c)
        c = best[1]
        unit_rank[u] = c
        on[c].append(u)
        tokens_cls[c] += ln[u]
    return unit_rank


def coschedule_score(unit_act, unit_len, expert_to_rank, unit_rank, D: int, w_load: int = 1, w_comm: int = 1):
    """what Alg. 1's outer loop compares: w_load * (the most tokens any cluster holds) + w_comm * (activation
    mass whose expert sits on another cluster than its unit: the all2all term of the Sec. 3.3 objective).
    Returns (score, max_tokens, remote_mass) as Python ints."""
    Q = np.asarray(unit_act, dtype=np.int64)
    U, E = Q.shape
    tokens = [0] * D
    remote = 0
    for u in range(U):
        tokens[int(unit_rank[u])] += int(unit_len[u])
        for e in range(E):
            if int(expert_to_rank[e]) != int(unit_rank[u]):
                remote += int(Q[u, e])
    return w_load * max(tokens) + w_comm * remote, max(tokens), remote


def coschedule(load, coact, unit_act, unit_len, D: int, alpha_e: int = 1, beta_e: int = 1, gamma_e: int = 0,
               alpha_r: int = 0, beta_r: int = 1, ft_passes: int = 8, n_steps: int = 4, w_load: int = 1,
               w_comm: int = 1):
    """The alternating co-clustering of Alg. 1 (App. B).  Start: the experts are placed with no unit scheduled
    (the request term is zero) and the units are clustered by their affinity to those experts (`unit_schedule`).
    Then n_steps times: place the experts for the current unit schedule, schedule the units for the new
    placement, score the pair; the pair of the lowest score is kept (equal -> the earlier step).
    Returns (expert_to_rank[E], unit_rank[U], step_score list of n_steps ints, best_step)."""
    assert n_steps >= 1
    e2r = expert_place_affinity(load, coact, D, None, None, alpha_e, 0, gamma_e, ft_passes)
    ur = unit_schedule(unit_act, unit_len, e2r, D, alpha_r, beta_r)
    best = None
    scores = []
    for step in range(n_steps):
        e2r = expert_place_affinity(load, coact, D, unit_act, ur, alpha_e, beta_e, gamma_e, ft_passes)
        ur = unit_schedule(unit_act, unit_len, e2r, D, alpha_r, beta_r)
        sc = coschedule_score(unit_act, unit_len, e2r, ur, D, w_load, w_comm)[0]
        scores.append(sc)
        if best is None or sc < best[0]:
            best = (sc, e2r.copy(), ur.copy(), step)
    return best[1], best[2], scores, best[3]


def token_labels(req_offsets, keys, req_rank, V: int, D: int, k: int):
    """The last lines of Alg. 1: count, per token id, how many of its occurrences sit in requests scheduled to
    each cluster; the token's label is the cluster of the highest count (equal -> smallest) and its confidence
    that count's share.  Same integer forms as `lookup_tables`: conf_q16 = floor(65536*share),
    level = round-half-up(k*share); an id that never occurs has dev = -1, conf_q16 = 0, level = 0.
    Returns (dev[V], conf_q16[V], level[V]) int32."""
    off = np.asarray(req_offsets)
    keys = np.asarray(keys)
    cnt = [[0] * D for _ in range(V)]
    for q in range(off.shape[0] - 1):
        for i in range(int(off[q]), int(off[q + 1])):
            v = int(keys[i])
            if 0 <= v < V:
                cnt[v][int(req_rank[q])] += 1
    dev = np.full(V, -1, dtype=np.int32)
    conf = np.zeros(V, dtype=np.int32)
    level = np.zeros(V, dtype=np.int32)
    for v in range(V):
        tot = sum(cnt[v])
        if tot == 0:
            continue
        best = max(range(D), key=lambda r: (cnt[v][r], -r))
        dev[v] = best
        conf[v] = (65536 * cnt[v][best]) // tot
        level[v] = (2 * k * cnt[v][best] + tot) // (2 * tot)
    return dev, conf, level


def home_assignment(T: int, D: int):
    """no reshuffle: tokens stay on their home rank; identity permutation"""
    tr = home_rank(T, D)
    idt = np.arange(T, dtype=np.int32)
    return tr, idt.copy(), idt.copy(), np.bincount(tr, minlength=D).astype(np.int32)


def local_pairs(ids, expert_to_rank, token_rank) -> int:
    """sum_i g[i, token_rank[i]]: pairs whose expert sits on the token's rank"""
    ids = np.asarray(ids)
    e2r = np.asarray(expert_to_rank)
    return int((e2r[ids] == np.asarray(token_rank)[:, None]).sum())


def reshuffle_bruteforce(ids, expert_to_rank, D: int, cap: int) -> int:
    """max over all capacity-feasible assignments of the local pair count (tiny inputs only)"""
    ids = np.asarray(ids)
    T = ids.shape[0]
    g = gain_matrix(ids, expert_to_rank, D)
    best = -1
    for assign in itertools.product(range(D), repeat=T):
        cnt = [0] * D
        ok = True
        for r in assign:
            cnt[r] += 1
            if cnt[r] > cap:
                ok = False
                break
        if ok:
            best = max(best, sum(int(g[i, assign[i]]) for i in range(T)))
    return best


def reshuffle_exact(ids, expert_to_rank, D: int, cap: int):
    """The assignment maximising local pairs under the capacity bound (the communication term of
    the Sec. 3.3 objective for a fixed placement), by min-cost flow: source -> token (cap 1) ->
    rank (cost -g[i,r]) -> sink (cap `cap`), successive shortest augmenting paths found with
    Bellman-Ford.  Returns (token_rank[T] int32, local_pair_count)."""
    ids = np.asarray(ids)
    T = ids.shape[0]
    assert cap * D >= T
    g = gain_matrix(ids, expert_to_rank, D)
    S, Z = T + D, T + D + 1
    n = T + D + 2
    # edge lists
    to, capa, cost, adj = [], [], [], [[] for _ in range(n)]

    def add(u, v, c, w):
        adj[u].append(len(to)); to.append(v); capa.append(c); cost.append(w)
        adj[v].append(len(to)); to.append(u); capa.append(0); cost.append(-w)

    for i in range(T):
        add(S, i, 1, 0)
        for r in range(D):
            add(i, T + r, 1, -int(g[i, r]))
    for r in range(D):
        add(T + r, Z, cap, 0)
    INF = 1 << 60
    total = 0
    for _ in range(T):
        dist = [INF] * n
        prev_e = [-1] * n
        dist[S] = 0
        inq = [False] * n
        queue = [S]
        inq[S] = True
        while queue:
            u = queue.pop(0)
            inq[u] = False
            for ei in adj[u]:
                if capa[ei] > 0 and dist[u] + cost[ei] < dist[to[ei]]:
                    dist[to[ei]] = dist[u] + cost[ei]
                    prev_e[to[ei]] = ei
                    if not inq[to[ei]]:
                        queue.append(to[ei]); inq[to[ei]] = True
        assert dist[Z] < INF
        v = Z
        while v != S:
            ei = prev_e[v]
            capa[ei] -= 1
            capa[ei ^ 1] += 1
            v = to[ei ^ 1]
        total += dist[Z]
    token_rank = np.zeros(T, dtype=np.int32)
    for i in range(T):
        for ei in adj[i]:
            if to[ei] >= T and to[ei] < T + D and ei % 2 == 0 and capa[ei] == 0:
                token_rank[i] = to[ei] - T
    return token_rank, -total


# --------------------------------------------------------------------------------------------
# a5  dispatch
# --------------------------------------------------------------------------------------------


def dispatch(X, ids, token_rank, inv_shf, phys_of_expert, D: int) -> Dict[str, np.ndarray]:
    """Dispatch half of expert parallelism (Sec. 1) on one device: order the P = T*k
    (token, expert) pairs by physical expert, pairs of one expert in arrival order of a
    rank-ordered all2all, i.e. by shuffled pair index p' = inv_shf[i]*k + j.
      slot                = position of (q, p') in the sort by q = phys_of_expert[ids[i,j]], then p'
      slot_of_pair[i*k+j] = slot;  pair_of_slot[slot] = i*k+j
      expert_offsets[q]   = first slot of physical expert q ([E] = P)
      rank_offsets[r]     = expert_offsets[r*m]
      X_perm[slot]        = X[i]
      send_matrix[s,r]    = #{(i,j): token_rank[i] = s and rank of ids[i,j] = r}
      remote_pairs        = sum_{s != r} send_matrix[s,r]   (dispatch direction only; the
                            all2all volume model alpha*k*B*S/G of Sec. 3.1 has
                            alpha = remote_pairs / P)"""
    ids = np.asarray(ids)
    T, k = ids.shape
    P = T * k
    phys = np.asarray(phys_of_expert, dtype=np.int64)
    E = phys.shape[0]
    m = E // D
    q = phys[ids].reshape(P)                                             # key of pair p
    pprime = (np.asarray(inv_shf, dtype=np.int64)[:, None] * k + np.arange(k)[None, :]).reshape(P)
    order = sorted(range(P), key=lambda p: (int(q[p]), int(pprime[p])))   # slot -> pair
    pair_of_slot = np.array(order, dtype=np.int64)
    slot_of_pair = np.zeros(P, dtype=np.int64)
    slot_of_pair[pair_of_slot] = np.arange(P)
    counts = np.bincount(q, minlength=E)
    expert_offsets = np.concatenate([[0], np.cumsum(counts)])
    rank_offsets = expert_offsets[::m].copy()
    send = np.zeros((D, D), dtype=np.int64)
    tr = np.asarray(token_rank, dtype=np.int64)
    for p in range(P):
        send[tr[p // k], q[p] // m] += 1
    remote = int(send.sum() - np.trace(send))
    out = dict(slot_of_pair=slot_of_pair.astype(np.int32), pair_of_slot=pair_of_slot.astype(np.int32),
               expert_offsets=expert_offsets.astype(np.int32), rank_offsets=rank_offsets.astype(np.int32),
               send_matrix=send.astype(np.uint32), remote_pairs=np.uint64(remote))
    if X is not None:
        out["X_perm"] = np.asarray(X)[pair_of_slot // k]
    return out


# --------------------------------------------------------------------------------------------
# a6  expert_ffn
# --------------------------------------------------------------------------------------------


def swiglu_ffn(x, W_gu, W_down) -> np.ndarray:
    """y = W_down ( silu(W_gate x) * (W_up x) ) for rows x[n,d]; W_gu[2F,d] = [gate; up],
    W_down[d,F]; fp64, no intermediate rounding."""
    x = np.asarray(x, dtype=np.float64)
    W_gu = np.asarray(W_gu, dtype=np.float64)
    F = W_gu.shape[0] // 2
    gate = x @ W_gu[:F].T
    up = x @ W_gu[F:].T
    h = gate / (1.0 + np.exp(-gate)) * up
    return h @ np.asarray(W_down, dtype=np.float64).T


def expert_ffn(X_perm, expert_offsets, expert_of_phys, weight_of, D: int, rank: int = -1, Y=None):
    """Grouped expert FFN (Sec. 2 "experts ... typically FFNs"; SwiGLU): for every physical
    expert q of `rank` (all ranks when -1), rows expert_offsets[q] .. expert_offsets[q+1] of
    X_perm go through the FFN of original expert expert_of_phys[q].  `weight_of(e)` returns
    (W_gu[e], W_down[e]).  Rows of other ranks are left as they are in Y."""
    Xp = np.asarray(X_perm)
    off = np.asarray(expert_offsets, dtype=np.int64)
    E = off.shape[0] - 1
    m = E // D
    Y = np.zeros(Xp.shape, dtype=np.float64) if Y is None else Y
    qs = range(E) if rank < 0 else range(rank * m, (rank + 1) * m)
    for q in qs:
        lo, hi = off[q], off[q + 1]
        if hi > lo:
            wgu, wdn = weight_of(int(expert_of_phys[q]))
            Y[lo:hi] = swiglu_ffn(Xp[lo:hi], wgu, wdn)
    return Y


# --------------------------------------------------------------------------------------------
# a7  combine
# --------------------------------------------------------------------------------------------


def combine(Y, slot_of_pair, topk_w, Y_shared=None) -> np.ndarray:
    """Out[i] = sum_j topk_w[i,j] * Y[slot_of_pair[i*k+j]] (+ Y_shared[i]); the combine all2all
    (Sec. 1) plus the un-permutation (`resume_tokens`, Alg. 3); fp64."""
    w = np.asarray(topk_w, dtype=np.float64)
    T, k = w.shape
    Y = np.asarray(Y, dtype=np.float64)
    s = np.asarray(slot_of_pair, dtype=np.int64).reshape(T, k)
    out = np.zeros((T, Y.shape[1]), dtype=np.float64)
    for j in range(k):
        out += w[:, j:j + 1] * Y[s[:, j]]
    if Y_shared is not None:
        out += np.asarray(Y_shared, dtype=np.float64)
    return out


# --------------------------------------------------------------------------------------------
# the plain definition the whole path must equal
# --------------------------------------------------------------------------------------------


def moe_definition(X, ids, topk_w, weight_of, shared=None, tokens=None) -> np.ndarray:
    """Out[i] = sum_j topk_w[i,j] * FFN_{ids[i,j]}(X[i]) (+ FFN_shared(X[i])), token by token from
    the definition, with no placement, shuffle or permutation.  `tokens` restricts to a sample."""
    X = np.asarray(X)
    ids = np.asarray(ids)
    w = np.asarray(topk_w, dtype=np.float64)
    toks = np.arange(X.shape[0]) if tokens is None else np.asarray(tokens)
    out = np.zeros((len(toks), X.shape[1]), dtype=np.float64)
    cache = {}
    for n, i in enumerate(toks):
        for j in range(ids.shape[1]):
            e = int(ids[i, j])
            if e not in cache:
                cache[e] = weight_of(e)
            out[n] += w[i, j] * swiglu_ffn(X[i:i + 1], *cache[e])[0]
        if shared is not None:
            out[n] += swiglu_ffn(X[i:i + 1], *shared)[0]
    return out


def moe_definition_by_expert(X, ids, topk_w, weight_of, shared=None, tokens=None) -> np.ndarray:
    """The same sum as `moe_definition`, taken expert by expert instead of token by token:
    Out[i] = sum over the experts e of (sum_j [ids[i,j] = e] topk_w[i,j]) * FFN_e(X[i]) (+ FFN_shared(X[i])),
    experts in ascending id, every expert's weights asked for exactly once (`weight_of(e)` is called for each
    expert some sampled token uses, in ascending order).  For layers whose experts do not fit host memory
    together.  Still no placement, shuffle or permutation; pinned to `moe_definition`."""
    X = np.asarray(X)
    ids = np.asarray(ids)
    w = np.asarray(topk_w, dtype=np.float64)
    toks = np.arange(X.shape[0]) if tokens is None else np.asarray(tokens)
    out = np.zeros((len(toks), X.shape[1]), dtype=np.float64)
    sub_ids = ids[toks]
    for e in np.unique(sub_ids):
        hit = sub_ids == e                                   # [n, k]
        rows = np.flatnonzero(hit.any(axis=1))
        coef = (w[toks[rows]] * hit[rows]).sum(axis=1)       # a token's experts are distinct: one term
        out[rows] += coef[:, None] * swiglu_ffn(X[toks[rows]], *weight_of(int(e)))
    if shared is not None:
        out += swiglu_ffn(X[toks], *shared)
    return out


# --------------------------------------------------------------------------------------------
# reported quantities
# --------------------------------------------------------------------------------------------


def remote_fraction(ids, expert_to_rank, token_rank) -> float:
    """alpha = remote pairs / (T*k); local activation rate LAR = 1 - alpha (Sec. 4.5)"""
    ids = np.asarray(ids)
    return 1.0 - local_pairs(ids, expert_to_rank, token_rank) / ids.size


def load_imbalance(send_matrix) -> float:
    """maximum rank load / median rank load over the pairs each rank computes (Sec. 4.6)"""
    col = np.asarray(send_matrix, dtype=np.float64).sum(axis=0)
    return float(col.max() / np.median(col))


def max_rel_err(a, b) -> float:
    """max|a-b| / max|b|: the tolerance measure for floating-point outputs"""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.abs(b).max()
    return float(np.abs(a - b).max() / den) if den > 0 else float(np.abs(a - b).max())
