#!/usr/bin/env python3
"""Benchmark of the semantic-parallel MoE layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME]

A step = one pass of the online hot path over one batch of seeded synthetic input that is already resident in
HBM:  route -> reshuffle -> dispatch (index + rows) -> expert_ffn (rank 0's experts) [-> shared expert on rank 0's
shard of tokens] -> combine.  The offline part (coact_hist on a profiling batch -> place on the host) runs once
before and is timed separately.

Without --config all five workloads run, each with W warm-up steps and exactly K timed steps of its own.  The
headline of the ONE JSON line that is printed is the largest workload that fits one GPU (the DeepSeek-V3-shaped
layer); the other four are sub-records under "configs", each with its ms/step, tokens/s, per-stage roofline
fractions, the roofline of its dominant stage and the CPU oracle timed on a bounded sample of the same workload.
With --config NAME only that workload runs and is the headline.
"""
import argparse
import glob
import json
import math
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
FP32_VECTOR_PEAK_TFLOPS = 157.3
HEADLINE = "c3_deepseek_v3"    # the largest of the five workloads; it fits one GPU (22.5 GB of expert weights)
NEXT_ROWS_ON = "c2_qwen3_30b"  # the workload the reports of the widened rows are quoted on


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(w, n_tokens, placement, weights, budget_s):
    """The oracle as it stands on a bounded sample: the first n_tokens of the batch through the whole chain, rank 0's
    FFN (+ the shared expert on the sample's first n_tokens / D tokens where the workload has one).  `placement` is
    the offline placement (an untimed input of the step); `weights` the numpy-drawn weights of rank 0's experts."""
    import numpy as np
    import workloads as WL
    from oracle import semmoe_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    X = WL.hidden(w)[:n_tokens]
    W_r, cb = WL.router_weight(w), WL.class_bias(w)
    tc = WL.token_class(w)[:n_tokens]
    e2r, phys, inv = placement
    shared = WL.shared_weight(w) if w.n_shared else None
    cap = -(-n_tokens // w.D)
    reps, dt = 0, 0.0
    while dt < budget_s and reps < 64:
        t0 = time.perf_counter()
        L = O.route_logits(X, W_r, None, tc, cb)
        ids, tw = O.select_topk(L, w.k, w.score, w.renorm, w.n_group, w.topk_group, w.routed_scale)
        tr, shf, ishf, rc = O.reshuffle(ids, e2r, w.D, cap)
        dsp = O.dispatch(X, ids, tr, ishf, phys, w.D)
        Y = O.expert_ffn(dsp["X_perm"], dsp["expert_offsets"], inv, lambda e: weights[e], w.D, rank=0)
        ysh = None
        if shared is not None:
            ysh = np.zeros((n_tokens, w.d))
            ysh[:cap] = O.swiglu_ffn(X[:cap], *shared)
        out = O.combine(Y, dsp["slot_of_pair"], tw, ysh)
        dt += time.perf_counter() - t0
        reps += 1
    assert out.shape == (n_tokens, w.d)
    return {"value": reps * n_tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "first %d tokens of the batch through the whole oracle chain (fp64 numpy; route, select, "
                      "reshuffle, dispatch, rank-0 expert FFN%s, combine), %d times over, %.1f s"
                      % (n_tokens, " + shared expert on %d tokens" % cap if shared is not None else "", reps, dt)}


def measured_traffic():
    """HBM bytes per launch of a stage from rocprofv3 counters, read from the committed summaries: every line
    `traffic_bytes <workload> <stage> <bytes>` of profiles/*.txt (FETCH_SIZE and WRITE_SIZE scaled by what the same
    counters read for a plain copy; the commands are in those files).  Counters cannot be read from inside a timed
    run, so the figures of the last profile are quoted; None where nothing was profiled."""
    out = {}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(path):
            p = line.split()
            if len(p) == 4 and p[0] == "traffic_bytes":
                out[(p[1], p[2])] = int(float(p[3]))
    return out


def achievable_peaks(m, torch, dev):
    """what this chip sustains on a plain device copy and on an MFMA-only loop (library probes), live"""
    def timed(fn, n):
        fn(); fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / n
    nbytes = 512 << 20   # read + written: 1 GiB, four times the Infinity Cache
    src = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    t_copy = timed(lambda: m.probe_copy(dst, src, nbytes), 10)
    words = torch.empty(2048 * 256, dtype=torch.int32, device=dev)
    t_read = timed(lambda: m.probe_stream(src, nbytes, 0, words), 10)
    t_write = timed(lambda: m.probe_stream(dst, nbytes, 1, words), 10)
    sink = torch.empty(256 * 256, dtype=torch.float32, device=dev)
    out = {"hbm_copy_GBps": round(2 * nbytes / t_copy / 1e9, 1), "hbm_read_only_GBps": round(nbytes / t_read / 1e9, 1),
           "hbm_write_only_GBps": round(nbytes / t_write / 1e9, 1)}
    iters = 20000
    for name, ops in (("constant", torch.ones(256 * 1024, dtype=torch.bfloat16, device=dev)),
                      ("random", torch.randn(256 * 1024, device=dev).to(torch.bfloat16))):
        flops = [0.0]
        def run():
            flops[0] = m.probe_mfma(ops, iters, sink)
        t = timed(run, 5)
        out["mfma_only_%s_operands_TFLOPs" % name] = round(flops[0] / t / 1e12, 1)
    # the K loop of the grouped GEMM's 256 x 256 tile alone (no tile list, epilogue or ragged edge; operands shared
    # in L2), whole and with parts taken out: what the loads and the LDS reads cost the MFMA stream
    n_panels, row_bytes, n_sl = 96, 16384, 2000
    panels = torch.randn(n_panels * 256 * row_bytes // 2, device=dev).to(torch.bfloat16)
    sink2 = torch.empty(256 * 512, dtype=torch.float32, device=dev)
    for v, name in ((0, "tile_loop"), (1, "tile_loop_without_loads"), (2, "tile_loop_without_lds_reads"),
                    (3, "tile_loop_mfma_and_barriers_only"), (4, "tile_loop_eight_waves")):
        flops = [0.0]
        def run():
            flops[0] = m.probe_tile_loop(panels, n_panels, row_bytes, v, n_sl, sink2)
        t = timed(run, 4)
        out[name + "_TFLOPs"] = round(flops[0] / t / 1e12, 1)
    del panels
    # the vendor library's plain square bf16 GEMM on random data (torch.matmul -> hipBLASLt / rocBLAS): a reference
    # for what a dense GEMM sustains on this chip, not part of the path
    n = 8192
    a = (torch.randn(n, n, device=dev) * 0.02).to(torch.bfloat16)
    b = torch.randn(n, n, device=dev).to(torch.bfloat16)
    c = torch.empty(n, n, dtype=torch.bfloat16, device=dev)
    t = timed(lambda: torch.matmul(a, b, out=c), 5)
    out["library_square_bf16_gemm_8192_TFLOPs"] = round(2.0 * n ** 3 / t / 1e12, 1)
    return out


def balance_study(args, w, m, up, X, W_r, tc, cb, ids, tw, load, coact, bufs, torch, np):
    T, D, P = w.T, w.D, w.P
    (token_rank, shf, inv_shf, rank_count, slot_of_pair, pair_of_slot, expert_offsets, rank_offsets, send_matrix,
     remote_pairs, X_perm, Y, W_gu, W_down) = bufs
    m.route(X, W_r, ids, tw, token_class=tc, class_bias=cb)
    load_h, coact_h = load.cpu().numpy().astype(np.uint64), coact.cpu().numpy().astype(np.uint64)

    def ffn_ms(rank, inv_s, reps=5):
        m.expert_ffn(rank, X_perm, expert_offsets, inv_s, W_gu, W_down, Y)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            m.expert_ffn(rank, X_perm, expert_offsets, inv_s, W_gu, W_down, Y)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    points = []
    for alpha, gamma, ft in ((1, 0, 8), (1, 0, 0), (16, 1, 0), (8, 1, 0), (4, 1, 0), (4, 1, 8), (2, 1, 0), (2, 1, 8),
                             (1, 1, 8), (1, 4, 8), (1, 16, 8), (1, 64, 8), (1, 256, 8), (0, 1, 0), (0, 1, 8)):
        e2r_s, phys_s, inv_s = (up(a) for a in m.place(load_h, coact_h, alpha, gamma, ft))
        rank_load = np.bincount(e2r_s.cpu().numpy(), weights=load_h.astype(np.float64), minlength=D)
        for cf in (1.0, 1.25, 1.5, 2.0, float(D)):
            cap = min(T, int(np.ceil(cf * T / D)))
            m.reshuffle(ids, e2r_s, token_rank, shf, inv_shf, rank_count, cap=cap)
            m.dispatch_index(ids, token_rank, shf, phys_s, slot_of_pair, pair_of_slot, expert_offsets,
                             rank_offsets, send_matrix, remote_pairs)
            m.dispatch_rows(X, slot_of_pair, X_perm)
            torch.cuda.synchronize()
            ro = rank_offsets.cpu().numpy()
            pairs = np.diff(ro)                       # pairs computed by each rank's experts
            tokens = rank_count.cpu().numpy()         # tokens held by each rank after the reshuffle
            per_rank = [ffn_ms(r, inv_s) for r in range(D)]
            points.append({
                "alpha": alpha, "gamma": gamma, "ft_passes": ft, "cf": round(cf, 2),
                "remote_pair_fraction": round(int(remote_pairs.item()) / P, 4),
                "pairs_per_rank_max_over_mean": round(float(pairs.max() / pairs.mean()), 3),
                "tokens_per_rank_max_over_mean": round(float(tokens.max() / tokens.mean()), 3),
                "profile_load_per_rank_max_over_mean": round(float(rank_load.max() / rank_load.mean()), 3),
                "ffn_ms_slowest_rank": round(max(per_rank), 4), "ffn_ms_mean_rank": round(float(np.mean(per_rank)), 4)})
    print(json.dumps({"study": "load balance: placement load weight x reshuffle capacity factor",
                      "config": {"workload": w.name, "T": T, "D": D, "E": w.E, "k": w.k}, "dtype": w.dtype,
                      "data": "synthetic", "points": points, "device": torch.cuda.get_device_name(0)}))


def run_config(name, args, traffic_tab):
    """one workload: set-up, offline placement, W warm-up + K timed steps, per-stage events, rooflines, CPU baseline"""
    import numpy as np
    import torch
    import workloads as WL
    import paper_2503_04398_amd as S

    dev = "cuda:0"
    w = WL.CONFIGS[name]
    adt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    b = 2 if w.dtype == "bf16" else 4
    T, d, E, k, F, D, P = w.T, w.d, w.E, w.k, w.F, w.D, w.P
    t_setup = time.time()

    def up(x, act=False):
        t = torch.from_numpy(np.ascontiguousarray(x)).to(dev)
        return t.to(adt) if act else t

    # ---------------- inputs, resident in HBM before anything is timed
    X = up(WL.hidden(w), True)
    W_r = up(WL.router_weight(w), True)
    tc = up(WL.token_class(w))
    cb = up(WL.class_bias(w))
    m = S.SemMoE(S.Config.from_workload(w), device=dev)
    i32 = dict(dtype=torch.int32, device=dev)
    ids = torch.empty(T, k, **i32)
    tw = torch.empty(T, k, dtype=torch.float32, device=dev)
    token_rank, shf, inv_shf = (torch.empty(T, **i32) for _ in range(3))
    rank_count = torch.empty(D, **i32)
    slot_of_pair, pair_of_slot = torch.empty(P, **i32), torch.empty(P, **i32)
    expert_offsets, rank_offsets = torch.empty(E + 1, **i32), torch.empty(D + 1, **i32)
    send_matrix = torch.empty(D, D, **i32)
    remote_pairs = torch.empty(1, dtype=torch.int64, device=dev)
    X_perm = torch.empty(P, d, dtype=adt, device=dev)
    Y = torch.zeros(P, d, dtype=adt, device=dev)
    Out = torch.empty(T, d, dtype=adt, device=dev)

    # ---------------- offline: profile batch -> co-activation histogram -> placement (host)
    Tp = w.profile_tokens
    mp = S.SemMoE(S.Config.from_workload(w, T=Tp, cap=-(-Tp // D)), device=dev)
    Xp = up(WL.hidden(w, profile=True), True)
    tcp = up(WL.token_class(w, profile=True))
    idp = torch.empty(Tp, k, **i32)
    twp = torch.empty(Tp, k, dtype=torch.float32, device=dev)
    load = torch.zeros(E, **i32)
    coact = torch.zeros(E, E, **i32)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    mp.route(Xp, W_r, idp, twp, token_class=tcp, class_bias=cb)
    mp.coact_hist(idp, Tp, load, coact)
    torch.cuda.synchronize()
    t_hist = time.perf_counter() - t0
    t0 = time.perf_counter()
    e2r_h, phys_h, inv_h = m.place(load.cpu().numpy().astype(np.uint64), coact.cpu().numpy().astype(np.uint64))
    t_place = time.perf_counter() - t0
    # token-to-expert activation table of the same profile batch -> schedule table (host)
    V = WL.vocab_size(w)
    keys_p = up(WL.token_key(w, profile=True))
    table = torch.zeros(V, E, **i32)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    mp.token_expert_hist(keys_p, idp, Tp, V, table)
    torch.cuda.synchronize()
    t_table = time.perf_counter() - t0
    t0 = time.perf_counter()
    sched_dev, sched_conf, sched_level = m.lookup_tables(table.cpu().numpy().view(np.uint32), e2r_h)
    t_lookup = time.perf_counter() - t0
    e2r, phys, inv = up(e2r_h), up(phys_h), up(inv_h)

    # ---------------- expert weights.  Rank 0's experts (the ones the timed FFN multiplies by, and the CPU baseline
    # too) and the shared expert come from the workload's numpy generator; the experts of the other ranks, which
    # only the all-ranks figure touches, are drawn on the device from the same distribution unless --host-weights.
    W_gu = torch.empty(E, 2 * F, d, dtype=adt, device=dev)
    W_down = torch.empty(E, d, F, dtype=adt, device=dev)
    rank0 = [int(inv_h[q]) for q in range(w.m)]
    host_experts = list(range(E)) if (args.host_weights or E * 3 * d * F <= (1 << 30)) else rank0
    weights0 = {}
    if args.zero_weights:
        W_gu.zero_()
        W_down.zero_()
    else:
        if len(host_experts) < E:
            g = torch.Generator(device=dev)
            g.manual_seed(w.seed + 17)
            for e in range(E):
                if e not in rank0:
                    W_gu[e].copy_((torch.randn(2 * F, d, generator=g, device=dev) * w.weight_std).to(adt))
                    W_down[e].copy_((torch.randn(d, F, generator=g, device=dev) * w.weight_std).to(adt))
        with ThreadPoolExecutor(max_workers=8) as pool:
            for e, (wgu, wdn) in zip(host_experts, pool.map(lambda e: WL.expert_weight(w, e), host_experts)):
                W_gu[e].copy_(up(wgu, True))
                W_down[e].copy_(up(wdn, True))
                if e in rank0:
                    weights0[e] = (wgu, wdn)
    n_sh = w.cap if w.n_shared else 0     # the shared expert's rows in the step: rank 0's shard of the tokens
    if w.n_shared:
        wgu, wdn = WL.shared_weight(w)
        W_gu_sh, W_down_sh = up(wgu, True), up(wdn, True)
        if args.zero_weights:
            W_gu_sh.zero_(); W_down_sh.zero_()
        Y_shared = torch.zeros(T, d, dtype=adt, device=dev)   # rows of the other ranks' shards stay zero
    say("[%s] set-up %.1f s (%d of %d experts from the numpy generator)" % (name, time.time() - t_setup, len(host_experts), E))

    bufs = (token_rank, shf, inv_shf, rank_count, slot_of_pair, pair_of_slot, expert_offsets, rank_offsets, send_matrix,
            remote_pairs, X_perm, Y, W_gu, W_down)
    if args.balance_study:
        balance_study(args, w, m, up, X, W_r, tc, cb, ids, tw, load, coact, bufs, torch, np)
        return None

    ffn_rank = -1 if args.all_ranks else 0
    stages = ["route", "reshuffle", "dispatch_index", "dispatch_rows", "expert_ffn"] + \
             (["shared_ffn"] if w.n_shared else []) + ["combine"]

    def step(ev=None):
        i = 0
        def mark():
            nonlocal i
            if ev: ev[i].record()
            i += 1
        mark()
        m.route(X, W_r, ids, tw, token_class=tc, class_bias=cb)
        mark()
        m.reshuffle(ids, e2r, token_rank, shf, inv_shf, rank_count)
        mark()
        m.dispatch_index(ids, token_rank, shf, phys, slot_of_pair, pair_of_slot, expert_offsets, rank_offsets,
                         send_matrix, remote_pairs)
        mark()
        m.dispatch_rows(X, slot_of_pair, X_perm)
        mark()
        m.expert_ffn(ffn_rank, X_perm, expert_offsets, inv, W_gu, W_down, Y)
        mark()
        if w.n_shared:
            m.shared_ffn(X, n_sh, W_gu_sh, W_down_sh, Y_shared)
            mark()
        m.combine(Y, slot_of_pair, tw, Out, Y_shared=Y_shared if w.n_shared else None)
        mark()

    # First K steps with HIP events (on the stream the kernels run on) between the calls: per-stage times.  The events
    # serialise the host side a little, so this loop is a few percent slower than the timed region below.  It also
    # brings the chip out of its idle clocks (they take some milliseconds of work to settle) before anything counts.
    for _ in range(max(args.warmup, 3)):
        step()
    torch.cuda.synchronize()
    n_ev = len(stages) + 1
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(events[s])
    torch.cuda.synchronize()
    ms_evented = (time.perf_counter() - t0) / args.steps * 1e3
    stage_ms = {nm: sum(ev[i].elapsed_time(ev[i + 1]) for ev in events) / args.steps for i, nm in enumerate(stages)}
    if args.calib_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)    # 256 MiB read + 256 MiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            m.probe_copy(dst, src, src.numel())
        torch.cuda.synchronize()
        del src, dst
    # W untimed warm-up steps, then the timed region: exactly K steps, nothing between the calls
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3
    ms_graph = None
    if args.graph:
        # one step captured in a HIP graph (the library only launches kernels: nothing in it is a memset node), then K
        # replays; replays are checked against the eager result, with eager work and syncs in between
        ref = Out.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step()
        for _ in range(3):
            Out.zero_()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(Out, ref), "graph replay differs from the eager step"
            step()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) / args.steps * 1e3
    # ---------------- the FFN of every rank's experts in one call (the whole device's expert work, not one rank's share)
    ms_ffn_all = float("nan")
    if not args.step_only:
        for _ in range(2):
            m.expert_ffn(-1, X_perm, expert_offsets, inv, W_gu, W_down, Y)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            m.expert_ffn(-1, X_perm, expert_offsets, inv, W_gu, W_down, Y)
        e1.record()
        torch.cuda.synchronize()
        ms_ffn_all = e0.elapsed_time(e1) / 5

    # ---------------- what the batch looked like
    ro = rank_offsets.cpu().numpy()
    eo = expert_offsets.cpu().numpy()
    rows_ffn = int(ro[D] - ro[0]) if args.all_ranks else int(ro[1] - ro[0])
    # the vendor library's dense GEMMs (torch.matmul) on the flops of the timed FFN launch, as if all its rows went to
    # one expert: [rows, d] x [d, 2F], then [rows, F] x [F, d].  No ragged groups, no SwiGLU, no tile left over at a
    # group's end: a reference from above for a grouped kernel on the same chip and data, not part of the path
    vendor = None
    if w.dtype == "bf16" and rows_ffn >= 128 * w.m and not args.step_only:   # not for decode shapes: one expert's weights
                                                                              # stay in cache, the launch streams them all
        e_ref = int(inv[0].item())
        A1, B1 = X_perm[:rows_ffn], W_gu[e_ref].t()
        C1 = torch.empty(rows_ffn, 2 * F, dtype=adt, device=dev)
        A2, B2 = C1[:, :F], W_down[e_ref].t()
        C2 = torch.empty(rows_ffn, d, dtype=adt, device=dev)
        def dense():
            torch.matmul(A1, B1, out=C1)
            torch.matmul(A2, B2, out=C2)
        for _ in range(3):
            dense()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            dense()
        e1.record()
        torch.cuda.synchronize()
        ms_dense = e0.elapsed_time(e1) / 10
        vendor = {"ms": round(ms_dense, 4), "TFLOP/s": round(6.0 * d * F * rows_ffn / (ms_dense * 1e-3) / 1e12, 1),
                  "what": "torch.matmul [rows,d]x[d,2F] + [rows,F]x[F,d] on the launch's rows, one expert's weights"}
        del C1, C2
    q_hi = E if args.all_ranks else w.m
    active = int((np.diff(eo[:q_hi + 1]) > 0).sum())       # experts of the FFN launch that hold at least one row
    remote = int(remote_pairs.item())
    send = send_matrix.cpu().numpy().astype(np.int64)
    col = send.sum(axis=0)
    # remote fraction of the same routing under vanilla placement + home ranks (index pass only)
    van = torch.arange(E, **i32)
    home = (torch.arange(T, device=dev) // (-(-T // D))).to(torch.int32)
    ident = torch.arange(T, **i32)
    rp2 = torch.empty(1, dtype=torch.int64, device=dev)
    tmp = [torch.empty_like(slot_of_pair) for _ in range(2)]
    m.dispatch_index(ids, home, ident, van, tmp[0], tmp[1], torch.empty_like(expert_offsets),
                     torch.empty_like(rank_offsets), torch.empty_like(send_matrix), rp2)
    rp3 = torch.empty(1, dtype=torch.int64, device=dev)
    m.dispatch_index(ids, home, ident, phys, tmp[0], tmp[1], torch.empty_like(expert_offsets),
                     torch.empty_like(rank_offsets), torch.empty_like(send_matrix), rp3)
    torch.cuda.synchronize()

    next_rows = None
    if name == NEXT_ROWS_ON and not (args.no_next_rows or args.step_only):
        # ---------------- next row: reshuffle with gain-aware spill rounds (not part of the timed step)
        rounds_report = {}
        for R in (2, 3, D):
            if str(R) in rounds_report:
                continue
            tr2, shf2, ish2 = (torch.empty(T, **i32) for _ in range(3))
            rc2 = torch.empty(D, **i32)
            for _ in range(3):
                m.reshuffle_rounds(ids, e2r, R, tr2, shf2, ish2, rc2)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                m.reshuffle_rounds(ids, e2r, R, tr2, shf2, ish2, rc2)
            e1.record()
            torch.cuda.synchronize()
            rpr = torch.empty(1, dtype=torch.int64, device=dev)
            m.dispatch_index(ids, tr2, shf2, phys, tmp[0], tmp[1], torch.empty_like(expert_offsets),
                             torch.empty_like(rank_offsets), torch.empty_like(send_matrix), rpr)
            torch.cuda.synchronize()
            rounds_report[str(R)] = {"ms": round(e0.elapsed_time(e1) / 20, 4),
                                     "remote_pair_fraction": round(int(rpr.item()) / P, 4)}

        # ---------------- the same refined to the optimum by moves of placed tokens (not part of the timed step)
        refine_report = {}
        if D <= 16 and w.k <= 15 and T <= 32768:
            info = torch.empty(2, **i32)
            for R in (1, 3):
                tr2, shf2, ish2 = (torch.empty(T, **i32) for _ in range(3))
                rc2 = torch.empty(D, **i32)
                for _ in range(2):
                    m.reshuffle_refine(ids, e2r, R, 1 << 30, tr2, shf2, ish2, rc2, info)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(10):
                    m.reshuffle_refine(ids, e2r, R, 1 << 30, tr2, shf2, ish2, rc2, info)
                e1.record()
                torch.cuda.synchronize()
                rpr = torch.empty(1, dtype=torch.int64, device=dev)
                m.dispatch_index(ids, tr2, shf2, phys, tmp[0], tmp[1], torch.empty_like(expert_offsets),
                                 torch.empty_like(rank_offsets), torch.empty_like(send_matrix), rpr)
                torch.cuda.synchronize()
                cyc, conv = (int(v) for v in info.cpu())
                refine_report["after_%d_round%s" % (R, "" if R == 1 else "s")] = {
                    "ms": round(e0.elapsed_time(e1) / 10, 4), "cycles": cyc, "optimal": bool(conv),
                    "remote_pair_fraction": round(int(rpr.item()) / P, 4)}

        # ---------------- next row: reshuffle from the schedule table, by token key alone (not part of the timed step)
        keys = up(WL.token_key(w))
        tabs = [up(t) for t in (sched_dev, sched_conf, sched_level)]
        lookup_report = {"vocabulary": V, "keys_seen_in_profile": int((sched_dev >= 0).sum())}
        for thr in (0, 16384, 32768):
            tr2, shf2, ish2 = (torch.empty(T, **i32) for _ in range(3))
            rc2 = torch.empty(D, **i32)
            for _ in range(3):
                m.reshuffle_lookup(keys, V, tabs[0], tabs[1], tabs[2], thr, tr2, shf2, ish2, rc2)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                m.reshuffle_lookup(keys, V, tabs[0], tabs[1], tabs[2], thr, tr2, shf2, ish2, rc2)
            e1.record()
            torch.cuda.synchronize()
            rpr = torch.empty(1, dtype=torch.int64, device=dev)
            m.dispatch_index(ids, tr2, shf2, phys, tmp[0], tmp[1], torch.empty_like(expert_offsets),
                             torch.empty_like(rank_offsets), torch.empty_like(send_matrix), rpr)
            torch.cuda.synchronize()
            lookup_report["thr_%.2f" % (thr / 65536)] = {
                "ms": round(e0.elapsed_time(e1) / 20, 4), "remote_pair_fraction": round(int(rpr.item()) / P, 4),
                "tokens_moved_off_home": int((tr2 != home).sum().item())}

        # ---------------- next row: Alg. 3 with both tables: the inter-layer device-sequence table A next to T.  The two
        # MoE layers before this one route the same tokens by their own router weights and class clusters; their
        # placements come from their own profile routing.  30 % of the tokens carry a key that all classes share.
        seq_p, seq_m = None, None
        t_seq = 0.0
        for layer in (2, 1):
            W_l, cb_l = up(WL.router_weight(w, layer), True), up(WL.class_bias(w, layer))
            id_l = torch.empty(Tp, k, **i32)
            mp.route(Xp, W_l, id_l, twp, token_class=tcp, class_bias=cb_l)
            ld_l, co_l = torch.zeros(E, **i32), torch.zeros(E, E, **i32)
            mp.coact_hist(id_l, Tp, ld_l, co_l)
            e2r_l = up(m.place(ld_l.cpu().numpy().astype(np.uint64), co_l.cpu().numpy().astype(np.uint64))[0])
            nxt = torch.empty(Tp, **i32)
            mp.device_sequence(id_l, e2r_l, Tp, seq_p, nxt)
            seq_p = nxt
            id_m = torch.empty(T, k, **i32)
            m.route(X, W_l, id_m, torch.empty_like(tw), token_class=tc, class_bias=cb_l)
            nxt = torch.empty(T, **i32)
            for _ in range(3):
                m.device_sequence(id_m, e2r_l, T, seq_m, nxt)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                m.device_sequence(id_m, e2r_l, T, seq_m, nxt)
            e1.record()
            torch.cuda.synchronize()
            t_seq = e0.elapsed_time(e1) / 20
            seq_m = nxt
        VA, VS = D * D, WL.vocab_size(w, shared=True)
        keys_sp, keys_sm = up(WL.token_key(w, profile=True, shared_frac=0.3)), up(WL.token_key(w, shared_frac=0.3))
        tab_t, tab_a = torch.zeros(VS, E, **i32), torch.zeros(VA, E, **i32)
        mp.token_expert_hist(keys_sp, idp, Tp, VS, tab_t)
        mp.token_expert_hist(seq_p, idp, Tp, VA, tab_a)
        torch.cuda.synchronize()
        tt = [up(t) for t in m.lookup_tables(tab_t.cpu().numpy().view(np.uint32), e2r_h)]
        ta = [up(t) for t in m.lookup_tables(tab_a.cpu().numpy().view(np.uint32), e2r_h)]
        none = [torch.full((1,), -1, **i32), torch.zeros(1, **i32), torch.zeros(1, **i32)]
        seq_report = {"look_back_layers": 2, "sequence_rows": VA, "rows_seen_in_profile": int((ta[0] >= 0).sum().item()),
                      "shared_key_share": 0.3, "device_sequence_ms": round(t_seq, 4)}
        for label, a_t, a_a in (("T_only", tt, none), ("A_only", none, ta), ("cond(T_p>A_p,T,A)", tt, ta)):
            tr2, shf2, ish2 = (torch.empty(T, **i32) for _ in range(3))
            rc2 = torch.empty(D, **i32)
            call = lambda: m.reshuffle_cond(keys_sm, a_t[0].shape[0], a_t[0], a_t[1], a_t[2], seq_m, a_a[0].shape[0],
                                            a_a[0], a_a[1], a_a[2], 0, tr2, shf2, ish2, rc2)
            for _ in range(3):
                call()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                call()
            e1.record()
            torch.cuda.synchronize()
            rpr = torch.empty(1, dtype=torch.int64, device=dev)
            m.dispatch_index(ids, tr2, shf2, phys, tmp[0], tmp[1], torch.empty_like(expert_offsets),
                             torch.empty_like(rank_offsets), torch.empty_like(send_matrix), rpr)
            torch.cuda.synchronize()
            seq_report[label] = {"ms": round(e0.elapsed_time(e1) / 20, 4),
                                 "remote_pair_fraction": round(int(rpr.item()) / P, 4),
                                 "tokens_moved_off_home": int((tr2 != home).sum().item())}

        # ---------------- next row: request-level scheduling (Attention-DP): requests = runs of tokens of one topic
        req_off_h, req_cls_h, req_key_h = WL.requests(w)
        n_req = len(req_off_h) - 1
        req_off, req_cls, req_key = up(req_off_h), up(req_cls_h), up(req_key_h)
        ids_r = torch.empty(T, k, **i32)
        tw_r = torch.empty(T, k, dtype=torch.float32, device=dev)
        m.route(X, W_r, ids_r, tw_r, token_class=req_cls, class_bias=cb)
        req_rank = torch.empty(n_req, **i32)
        tr2, shf2, ish2 = (torch.empty(T, **i32) for _ in range(3))
        rc2 = torch.empty(D, **i32)
        request_report = {"requests": n_req}
        for label, table_dev in (("round_robin", torch.full((V,), -1, **i32)), ("schedule_table", tabs[0])):
            for _ in range(3):
                m.request_schedule(req_off, n_req, req_key, V, table_dev, req_rank, tr2, shf2, ish2, rc2)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                m.request_schedule(req_off, n_req, req_key, V, table_dev, req_rank, tr2, shf2, ish2, rc2)
            e1.record()
            torch.cuda.synchronize()
            rpr = torch.empty(1, dtype=torch.int64, device=dev)
            m.dispatch_index(ids_r, tr2, shf2, phys, tmp[0], tmp[1], torch.empty_like(expert_offsets),
                             torch.empty_like(rank_offsets), torch.empty_like(send_matrix), rpr)
            torch.cuda.synchronize()
            rch = rc2.cpu().numpy()
            request_report[label] = {"ms": round(e0.elapsed_time(e1) / 20, 4),
                                     "remote_pair_fraction": round(int(rpr.item()) / P, 4),
                                     "tokens_per_rank_max_over_mean": round(float(rch.max() / max(rch.mean(), 1)), 3)}

        # ---------------- next row: the co-scheduling solver (Alg. 1 whole): profiling requests -> expert placement and
        # token labels together; judged by the remote-pair fraction of the measured batch's requests scheduled by Alg. 2
        pq_off_h, pq_cls_h, pq_key_h = WL.requests(w, profile=True)
        n_pq = len(pq_off_h) - 1
        idq = torch.empty(Tp, k, **i32)
        twq = torch.empty(Tp, k, dtype=torch.float32, device=dev)
        mp.route(Xp, W_r, idq, twq, token_class=up(pq_cls_h), class_bias=cb)
        unit_of = up(np.repeat(np.arange(n_pq), np.diff(pq_off_h)).astype(np.int32))
        unit_act = torch.zeros(n_pq, E, **i32)
        mp.token_expert_hist(unit_of, idq, Tp, n_pq, unit_act)
        load_q, coact_q, table_q = torch.zeros(E, **i32), torch.zeros(E, E, **i32), torch.zeros(V, E, **i32)
        mp.coact_hist(idq, Tp, load_q, coact_q)
        mp.token_expert_hist(up(pq_key_h), idq, Tp, V, table_q)
        torch.cuda.synchronize()
        load_qh, coact_qh = load_q.cpu().numpy().astype(np.uint64), coact_q.cpu().numpy().astype(np.uint64)
        act_h, table_qh = unit_act.cpu().numpy().astype(np.uint64), table_q.cpu().numpy().view(np.uint32)
        len_h = np.diff(pq_off_h).astype(np.uint64)
        pl_a = m.place(load_qh, coact_qh)
        t0 = time.perf_counter()
        cs = m.coschedule(load_qh, coact_qh, act_h, len_h, alpha_e=1, beta_e=1, gamma_e=0, alpha_r=0, beta_r=1,
                          ft_passes=8, n_steps=4, w_load=1, w_comm=1)
        t_cosched = time.perf_counter() - t0
        lab = m.token_labels(pq_off_h, pq_key_h, cs[3], V)
        cosched_report = {"profiling_requests": n_pq, "host_ms": round(t_cosched * 1e3, 3),
                          "step_score": [int(x) for x in cs[4]], "best_step": cs[5]}
        for label, pl, dev_tab in (("place+lookup_tables", pl_a, m.lookup_tables(table_qh, pl_a[0])[0]),
                                   ("coschedule+lookup_tables", cs, m.lookup_tables(table_qh, cs[0])[0]),
                                   ("coschedule+token_labels", cs, lab[0])):
            m.request_schedule(req_off, n_req, req_key, V, up(dev_tab), req_rank, tr2, shf2, ish2, rc2)
            rpr = torch.empty(1, dtype=torch.int64, device=dev)
            m.dispatch_index(ids_r, tr2, shf2, up(pl[1]), tmp[0], tmp[1], torch.empty_like(expert_offsets),
                             torch.empty_like(rank_offsets), torch.empty_like(send_matrix), rpr)
            torch.cuda.synchronize()
            rch = rc2.cpu().numpy()
            cosched_report[label] = {"remote_pair_fraction": round(int(rpr.item()) / P, 4),
                                     "tokens_per_rank_max_over_mean": round(float(rch.max() / max(rch.mean(), 1)), 3)}
        next_rows = {"reshuffle_with_spill_rounds": rounds_report, "reshuffle_refined_to_optimum": refine_report,
                     "reshuffle_from_schedule_table": lookup_report, "reshuffle_with_sequence_table": seq_report,
                     "request_schedule": request_report, "coschedule": cosched_report}
    del Xp, mp

    # ---------------- algorithmic bytes / flops per launch
    ffn_flops = 6.0 * d * F * rows_ffn
    # bytes the grouped FFN has to move at least: the weights of the experts that hold rows, every row in and out, the
    # hidden activation out and in again
    ffn_bytes = active * 3 * d * F * b + rows_ffn * (2 * d + 2 * F) * b
    ffn_hbm_bound = ffn_flops / ffn_bytes < MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9) / 4   # far below the ridge
    alg = {
        # the bf16 router is one fused kernel (logits never leave the chip); fp32 writes and re-reads them
        "route": ("hbm", T * d * b + E * d * b + T * k * 8 + (0 if w.dtype == "bf16" else 2 * 4 * T * E)),
        "reshuffle": ("hbm", T * k * 4 + E * 4 + 3 * T * 4),
        "dispatch_index": ("hbm", 2 * T * k * 4 + 2 * T * 4 + 2 * P * 4),
        "dispatch_rows": ("hbm", (T + P) * d * b + P * 4),
        "expert_ffn": (("alu" if w.dtype != "bf16" else ("hbm" if ffn_hbm_bound else "mfma")),
                       ffn_bytes if (w.dtype == "bf16" and ffn_hbm_bound) else ffn_flops),
        "shared_ffn": ("mfma", 6.0 * d * F * n_sh),
        "combine": ("hbm", (P + T) * d * b + P * 8 + (T * d * b if w.n_shared else 0)),
    }
    roof = {}
    for nm in stages:
        bound, work = alg[nm]
        sec = stage_ms[nm] * 1e-3
        if bound == "hbm":
            ach, peak, unit = work / sec / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, unit = work / sec / 1e12, "TFLOP/s"
            peak = MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else FP32_VECTOR_PEAK_TFLOPS
        roof[nm] = {"bound": bound, "achieved": round(ach, 2), "peak": peak, "unit": unit,
                    "frac": round(ach / peak, 4), "ms": round(stage_ms[nm], 4)}
    roof["expert_ffn"]["flops_frac_of_bf16_mfma_peak" if w.dtype == "bf16" else "flops_frac_of_fp32_vector_peak"] = round(
        ffn_flops / (stage_ms["expert_ffn"] * 1e-3) / 1e12 /
        (MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else FP32_VECTOR_PEAK_TFLOPS), 4)
    dominant = max(stages, key=lambda n: stage_ms[n])
    roofline = dict(roof[dominant])
    roofline.pop("ms")
    roofline = {kk: vv for kk, vv in roofline.items() if not kk.startswith("flops_frac")}
    roofline.update({"kernel": dominant + (" (gate/up + SwiGLU and down grouped GEMMs, one launch each)"
                                           if dominant == "expert_ffn" else ""),
                     "traffic": traffic_tab.get((name, dominant))})
    for nm in stages:
        if (name, nm) in traffic_tab:
            roof[nm]["traffic"] = traffic_tab[(name, nm)]

    rec = {
        "value": round(T / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "dtype": w.dtype,
        "config": {"workload": "%s: T=%d d=%d E=%d k=%d F=%d D=%d %s %s top-%d, semantic classes C=%d, expert FFN for %s%s"
                               % (w.name, T, d, E, k, F, D, w.dtype, w.score, k, w.C,
                                  "all ranks" if args.all_ranks else "rank 0's experts",
                                  " + the shared expert on rank 0's shard of %d tokens" % n_sh if w.n_shared else ""),
                   "cap": w.cap, "ffn_rows": rows_ffn, "ffn_experts_with_rows": active,
                   "ffn_rows_per_expert": [int(x) for x in np.diff(eo[:q_hi + 1])] if q_hi <= 32 else None},
        "roofline": roofline,
        "stages": roof,
        "expert_ffn_all_ranks": {"ms": round(ms_ffn_all, 4), "rows": P,
                                 ("TFLOP/s" if w.dtype == "bf16" else "TFLOP/s_fp32"): round(6.0 * d * F * P / (ms_ffn_all * 1e-3) / 1e12, 2),
                                 "frac": round(6.0 * d * F * P / (ms_ffn_all * 1e-3) / 1e12 /
                                               (MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else FP32_VECTOR_PEAK_TFLOPS), 4),
                                 "weights": "numpy generator" if len(host_experts) == E else
                                            "rank 0 numpy generator, other ranks drawn on the device"},
        "vendor_dense_gemms_same_flops": vendor,
        "ms_per_step_with_stage_events": round(ms_evented, 4),
        "ms_per_step_graph_replay": None if ms_graph is None else round(ms_graph, 4),
        "remote_pair_fraction": {"vanilla_placement_home_ranks": round(int(rp2.item()) / P, 4),
                                 "semmoe_placement_home_ranks": round(int(rp3.item()) / P, 4),
                                 "semmoe_placement_reshuffle": round(remote / P, 4)},
        "load_imbalance_max_over_median": round(float(col.max() / max(np.median(col), 1)), 4),
        "offline_ms": {"route+coact_hist(profile batch of %d)" % Tp: round(t_hist * 1e3, 3),
                       "place(host)": round(t_place * 1e3, 3),
                       "token_expert_hist(profile batch)": round(t_table * 1e3, 3),
                       "lookup_tables(host)": round(t_lookup * 1e3, 3)},
    }
    if next_rows:
        rec.update(next_rows)
    if args.step_only:
        rec.pop("expert_ffn_all_ranks")
    if not (args.no_cpu or args.zero_weights or args.step_only):
        t0 = time.time()
        rec["cpu_baseline"] = cpu_baseline(w, min(args.cpu_sample, T), (e2r_h, phys_h, inv_h), weights0, args.cpu_seconds)
        say("[%s] cpu baseline %.1f s" % (name, time.time() - t0))
    say("[%s] %.4f ms/step, %s" % (name, ms_per_step, ", ".join("%s %.1f us" % (n, stage_ms[n] * 1e3) for n in stages)))
    rec["_probe_handle"] = m
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default=None,
                    help="run this workload alone (default: all five, the largest as the headline, the others as sub-records)")
    ap.add_argument("--cpu-sample", type=int, default=2048, help="tokens of the CPU baseline's sample")
    ap.add_argument("--cpu-seconds", type=float, default=4.0, help="timed CPU work per workload, about")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true", help="skip the reports of the widened rows (spill rounds ...)")
    ap.add_argument("--no-peaks", action="store_true", help="skip the achievable-peak probes")
    ap.add_argument("--step-only", action="store_true",
                    help="nothing but set-up and the layer steps (for profiler runs: every launch of a step kernel in "
                         "the trace is then a launch of the step): no all-ranks FFN, widened rows, probes or CPU baseline")
    ap.add_argument("--all-ranks", action="store_true", help="FFN over every rank's experts instead of rank 0")
    ap.add_argument("--host-weights", action="store_true",
                    help="draw every expert's weights with the numpy generator (default: rank 0's experts and the shared "
                         "expert; the other ranks' experts, which the timed step never reads, on the device)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture one step in a HIP graph and time K replays (reported beside the eager figure)")
    ap.add_argument("--zero-weights", action="store_true",
                    help="diagnostic: expert weights all zero (same launches, tiles and bytes; shows how much of the GEMM "
                         "time depends on the data values, i.e. on power-limited clocks); the CPU baseline is skipped")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run the library's copy probe on 256 MiB three times between the loops: under rocprofv3 "
                         "--pmc its FETCH_SIZE / WRITE_SIZE readings give the scale of those counters")
    ap.add_argument("--balance-study", action="store_true",
                    help="instead of the timed layer step: sweep the load weight gamma of the placement and the capacity "
                         "factor of the reshuffle, and print remote-pair fraction, per-rank load imbalance and the FFN "
                         "time of the slowest rank for each point (one JSON line; workload: --config, default the "
                         "Qwen3-30B-shaped one)")
    ap.add_argument("--peaks-only", action="store_true",
                    help="only the library's probes (copy / read / write streams, MFMA-only loops, the tile's K loop whole "
                         "and in parts, the vendor GEMM): one JSON line; the command the counter profile of the probes runs")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is a one-GPU hot path (logical ranks are simulated on one device); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as WL

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.balance_study:
        run_config(args.config or NEXT_ROWS_ON, args, {})
        return
    if args.peaks_only:
        import paper_2503_04398_amd as S
        handle = S.SemMoE(S.Config(T=8, d=8, E=8, k=1, F=8, D=1, cap=8), allocate_workspace=False)
        print(json.dumps({"achievable": achievable_peaks(handle, torch, "cuda:0"), "data": "synthetic",
                          "device": torch.cuda.get_device_name(0)}))
        return
    traffic_tab = measured_traffic()
    names = [args.config] if args.config else [HEADLINE] + [n for n in WL.CONFIG_ORDER if n != HEADLINE]
    recs = {}
    for n in names:
        recs[n] = run_config(n, args, traffic_tab)
        torch.cuda.empty_cache()
    head = recs[names[0]]
    m = head.pop("_probe_handle")
    out = {"metric": "MoE-layer tokens/s on 1 MI355X", "value": head["value"], "unit": "tokens/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
           "config": head["config"], "roofline": head["roofline"]}
    for kk, vv in head.items():
        if kk not in out:
            out[kk] = vv
    cpu = out.pop("cpu_baseline", None)
    if len(names) > 1:
        out["configs"] = {}
        for n in names[1:]:
            r = recs[n]
            r.pop("_probe_handle", None)
            out["configs"][n] = r
    out["device"] = torch.cuda.get_device_name(0)
    if not (args.no_peaks or args.step_only):
        out["achievable"] = achievable_peaks(m, torch, "cuda:0")
        # each MFMA-bound FFN stage against what this chip, in this run, gave the K loop of its own tile with every
        # load hitting in L2 (no ragged groups, no epilogue, no tail): the share of the loop's rate that survives them
        loop = out["achievable"].get("tile_loop_TFLOPs")
        for r in [out] + list(out.get("configs", {}).values()):
            for nm in ("expert_ffn", "shared_ffn"):
                st = r.get("stages", {}).get(nm)
                if st and st.get("bound") == "mfma" and st.get("unit") == "TFLOP/s" and r.get("dtype") == "bf16" and loop:
                    st["frac_of_measured_tile_loop"] = round(st["achieved"] / loop, 4)
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
