"""Shared plumbing of the GPU parity tests: upload seeded inputs, run the HIP path through the C ABI
binding, read results back as numpy, and run the oracle chain on the same inputs.

Parity chain: the router GEMM's accumulation order differs between CPU and MFMA, so the oracle's
selection runs on the GPU's fp32 logits (after those were checked against the oracle's own logits);
every later integer stage of the oracle runs on those ids and is compared bit for bit.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
import torch

import workloads as WL
from oracle import semmoe_oracle as O
import paper_2503_04398_amd as S

TOL = {"fp32": 1e-5, "bf16": 2e-2}     # max|a-b| / max|b|, the tolerance the target states
DEV = "cuda:0"


def act_dtype(w):
    return torch.bfloat16 if w.dtype == "bf16" else torch.float32


def to_dev(x: np.ndarray, w=None):
    t = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    if w is not None and t.dtype == torch.float32 and w.dtype == "bf16":
        t = t.to(torch.bfloat16)          # exact: the generators only emit bf16-representable values
    return t


def to_np(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.detach().cpu().numpy()


@dataclass
class Inputs:
    w: WL.Workload
    X: np.ndarray
    W_r: np.ndarray
    token_class: np.ndarray
    class_bias: np.ndarray


def make_inputs(w: WL.Workload, profile: bool = False, n: Optional[int] = None) -> Inputs:
    return Inputs(w, WL.hidden(w, profile, n), WL.router_weight(w), WL.token_class(w, profile, n), WL.class_bias(w))


class Layer:
    """Device buffers of one layer + the HIP path, call by call."""

    def __init__(self, w: WL.Workload, cap: Optional[int] = None, T: Optional[int] = None):
        self.w = w
        self.T = w.T if T is None else T
        self.cfg = S.Config.from_workload(w, cap=cap if cap is not None else -(-self.T // w.D), T=self.T)
        self.m = S.SemMoE(self.cfg, device=DEV)
        T_, k, E, D = max(self.T, 1), w.k, w.E, w.D      # zero-size tensors have a null pointer
        i32 = dict(dtype=torch.int32, device=DEV)
        self.logits = torch.empty(T_, E, dtype=torch.float32, device=DEV)
        self.ids = torch.empty(T_, k, **i32)
        self.tw = torch.empty(T_, k, dtype=torch.float32, device=DEV)
        self.token_rank = torch.empty(T_, **i32)
        self.shf = torch.empty(T_, **i32)
        self.inv_shf = torch.empty(T_, **i32)
        self.rank_count = torch.empty(D, **i32)
        self.slot_of_pair = torch.empty(T_ * k, **i32)
        self.pair_of_slot = torch.empty(T_ * k, **i32)
        self.expert_offsets = torch.empty(E + 1, **i32)
        self.rank_offsets = torch.empty(D + 1, **i32)
        self.send_matrix = torch.empty(D, D, **i32)
        self.remote_pairs = torch.empty(1, dtype=torch.int64, device=DEV)

    # ---- route
    def route(self, inp: Inputs, b_g=None, sel_bias=None):
        w = self.w
        self.X = to_dev(inp.X, w)
        self.W_r = to_dev(inp.W_r, w)
        self.tc = to_dev(inp.token_class)
        self.cb = to_dev(inp.class_bias)
        self.m.route(self.X, self.W_r, self.ids, self.tw, b_g=None if b_g is None else to_dev(b_g),
                     token_class=self.tc, class_bias=self.cb, sel_bias=None if sel_bias is None else to_dev(sel_bias),
                     logits_out=self.logits)
        torch.cuda.synchronize()
        return to_np(self.logits), to_np(self.ids), to_np(self.tw)

    def set_routing(self, ids: np.ndarray, tw: Optional[np.ndarray] = None):
        self.ids.copy_(torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)))
        if tw is not None:
            self.tw.copy_(torch.from_numpy(np.ascontiguousarray(tw, dtype=np.float32)))

    # ---- histogram + placement
    def profile_placement(self, ids_dev: torch.Tensor, alpha=1, gamma=0, ft_passes=8):
        E = self.w.E
        load = torch.zeros(E, dtype=torch.int32, device=DEV)
        coact = torch.zeros(E, E, dtype=torch.int32, device=DEV)
        self.m.coact_hist(ids_dev, ids_dev.shape[0], load, coact)
        torch.cuda.synchronize()
        load_np = to_np(load).astype(np.uint64)
        coact_np = to_np(coact).astype(np.uint64)
        return load_np, coact_np, self.m.place(load_np, coact_np, alpha, gamma, ft_passes)

    def set_placement(self, e2r, phys, inv):
        self.e2r = to_dev(np.asarray(e2r, dtype=np.int32))
        self.phys = to_dev(np.asarray(phys, dtype=np.int32))
        self.inv = to_dev(np.asarray(inv, dtype=np.int32))

    # ---- reshuffle
    def reshuffle(self, cap=None):
        self.m.reshuffle(self.ids, self.e2r, self.token_rank, self.shf, self.inv_shf, self.rank_count, cap=cap)
        torch.cuda.synchronize()
        return tuple(to_np(t) for t in (self.token_rank, self.shf, self.inv_shf, self.rank_count))

    def reshuffle_rounds(self, rounds, cap=None):
        self.m.reshuffle_rounds(self.ids, self.e2r, rounds, self.token_rank, self.shf, self.inv_shf, self.rank_count,
                                cap=cap)
        torch.cuda.synchronize()
        return tuple(to_np(t) for t in (self.token_rank, self.shf, self.inv_shf, self.rank_count))

    def reshuffle_refine(self, rounds=1, max_cycles=1 << 30, cap=None):
        """returns ((token_rank, shf, inv_shf, rank_count), cycles, converged)"""
        info = torch.full((2,), -7, dtype=torch.int32, device=DEV)
        self.m.reshuffle_refine(self.ids, self.e2r, rounds, max_cycles, self.token_rank, self.shf, self.inv_shf,
                                self.rank_count, info, cap=cap)
        torch.cuda.synchronize()
        cyc, conv = (int(v) for v in to_np(info))
        return tuple(to_np(t) for t in (self.token_rank, self.shf, self.inv_shf, self.rank_count)), cyc, conv

    def token_expert_hist(self, keys, ids, V, table=None):
        """accumulate one batch into the activation table; returns the device table (int32 storage of the u32 counts)"""
        if table is None:
            table = torch.zeros(V, self.w.E, dtype=torch.int32, device=DEV)
        keys_d = to_dev(np.asarray(keys, dtype=np.int32))
        ids_d = to_dev(np.asarray(ids, dtype=np.int32))
        self.m.token_expert_hist(keys_d, ids_d, ids_d.shape[0], V, table)
        torch.cuda.synchronize()
        return table

    def reshuffle_lookup(self, keys, dev, conf_q16, level, thr_q16, cap=None):
        keys_d = to_dev(np.asarray(keys, dtype=np.int32))
        tabs = [to_dev(np.asarray(t, dtype=np.int32)) for t in (dev, conf_q16, level)]
        self.m.reshuffle_lookup(keys_d, tabs[0].shape[0], tabs[0], tabs[1], tabs[2], thr_q16, self.token_rank,
                                self.shf, self.inv_shf, self.rank_count, cap=cap)
        torch.cuda.synchronize()
        return tuple(to_np(t) for t in (self.token_rank, self.shf, self.inv_shf, self.rank_count))

    def reshuffle_cond(self, keys, tabs_t, seq_keys, tabs_a, thr_q16, cap=None):
        keys_d = to_dev(np.asarray(keys, dtype=np.int32))
        seq_d = to_dev(np.asarray(seq_keys, dtype=np.int32))
        tt = [to_dev(np.asarray(t, dtype=np.int32)) for t in tabs_t]
        ta = [to_dev(np.asarray(t, dtype=np.int32)) for t in tabs_a]
        self.m.reshuffle_cond(keys_d, tt[0].shape[0], tt[0], tt[1], tt[2], seq_d, ta[0].shape[0], ta[0], ta[1], ta[2],
                              thr_q16, self.token_rank, self.shf, self.inv_shf, self.rank_count, cap=cap)
        torch.cuda.synchronize()
        return tuple(to_np(t) for t in (self.token_rank, self.shf, self.inv_shf, self.rank_count))

    def device_sequence(self, ids, e2r, seq_in=None):
        ids_d = to_dev(np.asarray(ids, dtype=np.int32))
        n = ids_d.shape[0]
        out = torch.full((max(n, 1),), -9, dtype=torch.int32, device=DEV)
        seq_d = None if seq_in is None else to_dev(np.asarray(seq_in, dtype=np.int32))
        self.m.device_sequence(ids_d, to_dev(np.asarray(e2r, dtype=np.int32)), n, seq_d, out)
        torch.cuda.synchronize()
        return to_np(out)[:n]

    def request_schedule(self, req_offsets, keys, dev):
        off_d = to_dev(np.asarray(req_offsets, dtype=np.int32))
        keys_d = to_dev(np.asarray(keys, dtype=np.int32))
        dev_d = to_dev(np.asarray(dev, dtype=np.int32))
        n_req = off_d.shape[0] - 1
        req_rank = torch.full((max(n_req, 1),), -7, dtype=torch.int32, device=DEV)
        self.m.request_schedule(off_d, n_req, keys_d, dev_d.shape[0], dev_d, req_rank, self.token_rank, self.shf,
                                self.inv_shf, self.rank_count)
        torch.cuda.synchronize()
        return (to_np(req_rank)[:n_req],) + tuple(
            to_np(t) for t in (self.token_rank, self.shf, self.inv_shf, self.rank_count))

    def set_assignment(self, token_rank, shf, inv_shf):
        self.token_rank.copy_(torch.from_numpy(np.asarray(token_rank, dtype=np.int32)))
        self.shf.copy_(torch.from_numpy(np.asarray(shf, dtype=np.int32)))
        self.inv_shf.copy_(torch.from_numpy(np.asarray(inv_shf, dtype=np.int32)))

    # ---- dispatch
    def dispatch(self, with_rows=True):
        w = self.w
        if with_rows:
            self.X_perm = torch.empty(self.T * w.k, w.d, dtype=act_dtype(w), device=DEV)
        self.m.dispatch(self.X if with_rows else None, self.ids, self.token_rank, self.shf, self.phys,
                        self.X_perm if with_rows else None, self.slot_of_pair, self.pair_of_slot,
                        self.expert_offsets, self.rank_offsets, self.send_matrix, self.remote_pairs)
        torch.cuda.synchronize()
        out = dict(slot_of_pair=to_np(self.slot_of_pair), pair_of_slot=to_np(self.pair_of_slot),
                   expert_offsets=to_np(self.expert_offsets), rank_offsets=to_np(self.rank_offsets),
                   send_matrix=to_np(self.send_matrix).astype(np.uint32),
                   remote_pairs=np.uint64(int(self.remote_pairs.item())))
        return out

    # ---- expert weights
    def load_experts(self, experts):
        """device W_gu[E,2F,d], W_down[E,d,F]; only `experts` are filled (the rest stays unread)"""
        w = self.w
        if not hasattr(self, "W_gu"):
            self.W_gu = torch.empty(w.E, 2 * w.F, w.d, dtype=act_dtype(w), device=DEV)
            self.W_down = torch.empty(w.E, w.d, w.F, dtype=act_dtype(w), device=DEV)
            self._loaded = set()
        for e in experts:
            e = int(e)
            if e not in self._loaded:
                wgu, wdn = WL.expert_weight(w, e)
                self.W_gu[e].copy_(to_dev(wgu, w))
                self.W_down[e].copy_(to_dev(wdn, w))
                self._loaded.add(e)

    def expert_ffn(self, rank, poison: Optional[float] = None):
        w = self.w
        self.Y = torch.empty(self.T * w.k, w.d, dtype=act_dtype(w), device=DEV)
        if poison is not None:
            self.Y.fill_(poison)
        self.m.expert_ffn(rank, self.X_perm, self.expert_offsets, self.inv, self.W_gu, self.W_down, self.Y)
        torch.cuda.synchronize()
        return self.Y

    def shared_ffn(self):
        w = self.w
        wgu, wdn = WL.shared_weight(w)
        self.W_gu_sh, self.W_down_sh = to_dev(wgu, w), to_dev(wdn, w)
        self.Y_shared = torch.empty(self.T, w.d, dtype=act_dtype(w), device=DEV)
        self.m.shared_ffn(self.X, self.T, self.W_gu_sh, self.W_down_sh, self.Y_shared)
        torch.cuda.synchronize()
        return self.Y_shared

    def combine(self, Y=None, Y_shared=None):
        w = self.w
        self.Out = torch.empty(self.T, w.d, dtype=act_dtype(w), device=DEV)
        self.m.combine(self.Y if Y is None else Y, self.slot_of_pair, self.tw, self.Out, Y_shared=Y_shared)
        torch.cuda.synchronize()
        return to_np(self.Out)


def oracle_select(w: WL.Workload, logits: np.ndarray, sel_bias=None):
    return O.select_topk(logits, w.k, w.score, w.renorm, w.n_group, w.topk_group, w.routed_scale, sel_bias)


def assert_close(got, want, dtype: str, what: str = ""):
    err = O.max_rel_err(got, want)
    assert err <= TOL[dtype], "%s: max|a-b|/max|b| = %.3e > %.1e" % (what, err, TOL[dtype])
    return err
