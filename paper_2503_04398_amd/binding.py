"""ctypes binding of libsemmoe.so: argument marshalling only.

Every step of the path runs inside the library's HIP kernels; this module turns torch tensors into
raw pointers, passes torch's current stream, and raises on a non-zero status.  torch is used for
device memory and streams, nothing else.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))

STATUS_NAMES = {0: "OK", -1: "EINVAL", -2: "ESHAPE", -3: "EWORKSPACE", -4: "EHIP", -5: "EUNSUPPORTED"}
FP32, BF16 = 0, 1
SOFTMAX, SIGMOID = 0, 1


class SemMoEError(RuntimeError):
    def __init__(self, call: str, status: int, hip_error: int = 0):
        self.call, self.status, self.hip_error = call, status, hip_error
        msg = "%s failed: %s (%d)" % (call, STATUS_NAMES.get(status, "?"), status)
        if status == -4:
            msg += ", hipError_t %d" % hip_error
        super().__init__(msg)


class _CConfig(C.Structure):
    _fields_ = [("T", C.c_int32), ("d", C.c_int32), ("E", C.c_int32), ("k", C.c_int32), ("F", C.c_int32),
                ("D", C.c_int32), ("dtype", C.c_int32), ("score", C.c_int32), ("renorm", C.c_int32),
                ("n_group", C.c_int32), ("topk_group", C.c_int32), ("routed_scale", C.c_float),
                ("cap", C.c_int32), ("num_classes", C.c_int32)]


class CoschedParams(C.Structure):
    """semmoe_cosched_params of the C header, field for field"""
    _fields_ = [("alpha_e", C.c_int64), ("beta_e", C.c_int64), ("gamma_e", C.c_int64), ("alpha_r", C.c_int64),
                ("beta_r", C.c_int64), ("w_load", C.c_int64), ("w_comm", C.c_int64), ("ft_passes", C.c_int32),
                ("n_steps", C.c_int32)]


@dataclass
class Config:
    T: int
    d: int
    E: int
    k: int
    F: int
    D: int
    dtype: int = BF16
    score: int = SOFTMAX
    renorm: bool = True
    n_group: int = 1
    topk_group: int = 1
    routed_scale: float = 1.0
    cap: int = 0
    num_classes: int = 0

    def __post_init__(self):
        # the names of the workload descriptions are accepted for the two enumerations
        if isinstance(self.dtype, str):
            if self.dtype not in ("bf16", "fp32"):
                raise ValueError("dtype must be 'bf16' or 'fp32' (or the BF16 / FP32 constants)")
            self.dtype = BF16 if self.dtype == "bf16" else FP32
        if isinstance(self.score, str):
            if self.score not in ("softmax", "sigmoid"):
                raise ValueError("score must be 'softmax' or 'sigmoid' (or the SOFTMAX / SIGMOID constants)")
            self.score = SIGMOID if self.score == "sigmoid" else SOFTMAX

    def c(self) -> _CConfig:
        return _CConfig(self.T, self.d, self.E, self.k, self.F, self.D, self.dtype, self.score, int(self.renorm),
                        self.n_group, self.topk_group, self.routed_scale, self.cap, self.num_classes)

    @staticmethod
    def from_workload(w, cap: Optional[int] = None, T: Optional[int] = None) -> "Config":
        return Config(T=w.T if T is None else T, d=w.d, E=w.E, k=w.k, F=w.F, D=w.D,
                      dtype=BF16 if w.dtype == "bf16" else FP32,
                      score=SIGMOID if w.score == "sigmoid" else SOFTMAX, renorm=bool(w.renorm),
                      n_group=w.n_group, topk_group=w.topk_group, routed_scale=w.routed_scale,
                      cap=w.cap if cap is None else cap, num_classes=w.C)


def lib_path() -> str:
    return os.environ.get("SEMMOE_LIB", os.path.join(HERE, "lib", "libsemmoe.so"))


_LIB = None
_P = C.c_void_p
_SIGS = {
    "semmoe_version": ([], C.c_int32),
    "semmoe_last_hip_error": ([], C.c_int32),
    "semmoe_workspace_bytes": ([_P, C.POINTER(C.c_size_t)], C.c_int32),
    "semmoe_set_tuning": ([C.c_int32, C.c_int32], C.c_int32),
    "semmoe_get_tuning": ([C.c_int32, _P], C.c_int32),
    "semmoe_route": ([_P] * 12 + [C.c_size_t], C.c_int32),
    "semmoe_route_from_logits": ([_P] * 6, C.c_int32),
    "semmoe_coact_hist": ([_P, _P, _P, C.c_int32, _P, _P], C.c_int32),
    "semmoe_token_expert_hist": ([_P, _P, _P, _P, C.c_int32, C.c_int32, _P], C.c_int32),
    "semmoe_lookup_tables": ([_P, _P, _P, C.c_int32, _P, _P, _P], C.c_int32),
    "semmoe_place": ([_P, _P, _P, C.c_int64, C.c_int64, C.c_int32, _P, _P, _P], C.c_int32),
    "semmoe_coschedule": ([_P, _P, _P, _P, _P, C.c_int32, _P, _P, _P, _P, _P, _P, _P], C.c_int32),
    "semmoe_token_labels": ([_P, _P, C.c_int32, _P, _P, C.c_int32, _P, _P, _P], C.c_int32),
    "semmoe_reshuffle": ([_P] * 9 + [C.c_size_t], C.c_int32),
    "semmoe_reshuffle_static": ([_P] * 8, C.c_int32),
    "semmoe_reshuffle_rounds": ([_P] * 4 + [C.c_int32] + [_P] * 5 + [C.c_size_t], C.c_int32),
    "semmoe_reshuffle_refine": ([_P] * 4 + [C.c_int32, C.c_int32] + [_P] * 6 + [C.c_size_t], C.c_int32),
    "semmoe_reshuffle_lookup": ([_P, _P, _P, C.c_int32, _P, _P, _P, C.c_int32] + [_P] * 5 + [C.c_size_t], C.c_int32),
    "semmoe_reshuffle_cond": ([_P, _P, _P, C.c_int32, _P, _P, _P, _P, C.c_int32, _P, _P, _P, C.c_int32] + [_P] * 5
                              + [C.c_size_t], C.c_int32),
    "semmoe_device_sequence": ([_P, _P, _P, _P, C.c_int32, _P, _P], C.c_int32),
    "semmoe_request_schedule": ([_P, _P, _P, C.c_int32, _P, C.c_int32] + [_P] * 7 + [C.c_size_t], C.c_int32),
    "semmoe_dispatch": ([_P] * 15 + [C.c_size_t], C.c_int32),
    "semmoe_dispatch_index": ([_P] * 13 + [C.c_size_t], C.c_int32),
    "semmoe_dispatch_rows": ([_P] * 5, C.c_int32),
    "semmoe_expert_ffn": ([_P, _P, C.c_int32] + [_P] * 7 + [C.c_size_t], C.c_int32),
    "semmoe_shared_ffn": ([_P, _P, _P, C.c_int32, _P, _P, _P, _P, C.c_size_t], C.c_int32),
    "semmoe_combine": ([_P] * 7, C.c_int32),
    "semmoe_probe_copy": ([_P, _P, _P, C.c_size_t], C.c_int32),
    "semmoe_probe_stream": ([_P, _P, C.c_size_t, C.c_int32, _P], C.c_int32),
    "semmoe_probe_mfma": ([_P, _P, C.c_int32, _P, C.POINTER(C.c_double)], C.c_int32),
    "semmoe_probe_tile_loop": ([_P, _P, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _P, C.POINTER(C.c_double)], C.c_int32),
}
EXPORTS = tuple(_SIGS)


def load_library():
    """Load libsemmoe.so (built by `python -m paper_2503_04398_amd.build`).  No fallback."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise SemMoEError("load_library: %s is missing; build it with "
                              "`python -m paper_2503_04398_amd.build`" % path, -1)
        lib = C.CDLL(path)
        for name, (args, res) in _SIGS.items():
            fn = getattr(lib, name)
            fn.argtypes, fn.restype = args, res
        _LIB = lib
    return _LIB


def _ptr(t):
    """device (or host) pointer of a torch tensor / numpy array / None / int"""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        assert t.is_contiguous(), "tensors must be contiguous"
        return t.data_ptr()
    return t.ctypes.data


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None


class SemMoE:
    """One config + one workspace; methods mirror the C entry points one to one."""

    def __init__(self, cfg: Config, device="cuda:0", allocate_workspace: bool = True):
        self.lib = load_library()
        self.cfg = cfg
        self.device = device
        self.ws = None
        self.ws_bytes = 0
        self.ws_shared = None
        if allocate_workspace:
            import torch
            self.ws_bytes = self.workspace_bytes()
            self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)

    # -- helpers
    def _check(self, name: str, st: int):
        if st != 0:
            raise SemMoEError(name, st, self.lib.semmoe_last_hip_error())

    def _cfg(self, **over):
        c = self.cfg.c()
        for k_, v in over.items():
            setattr(c, k_, v)
        return c

    def workspace_bytes(self) -> int:
        n = C.c_size_t(0)
        c = self._cfg()
        self._check("semmoe_workspace_bytes", self.lib.semmoe_workspace_bytes(C.byref(c), C.byref(n)))
        return int(n.value)

    def set_tuning(self, key: int, value: int):
        self._check("semmoe_set_tuning", self.lib.semmoe_set_tuning(int(key), int(value)))

    def get_tuning(self, key: int) -> int:
        v = C.c_int32(0)
        self._check("semmoe_get_tuning", self.lib.semmoe_get_tuning(int(key), C.byref(v)))
        return int(v.value)

    # -- entry points
    def route(self, X, W_r, topk_ids, topk_w, b_g=None, token_class=None, class_bias=None, sel_bias=None,
              logits_out=None, T=None):
        c = self._cfg(**({"T": T} if T is not None else {}))
        self._check("semmoe_route", self.lib.semmoe_route(
            C.byref(c), _stream(), _ptr(X), _ptr(W_r), _ptr(b_g), _ptr(token_class), _ptr(class_bias),
            _ptr(sel_bias), _ptr(logits_out), _ptr(topk_ids), _ptr(topk_w), _ptr(self.ws), self.ws_bytes))

    def route_from_logits(self, logits, topk_ids, topk_w, sel_bias=None, T=None):
        c = self._cfg(**({"T": T} if T is not None else {}))
        self._check("semmoe_route_from_logits", self.lib.semmoe_route_from_logits(
            C.byref(c), _stream(), _ptr(logits), _ptr(sel_bias), _ptr(topk_ids), _ptr(topk_w)))

    def coact_hist(self, topk_ids, T_batch, load, coact):
        c = self._cfg()
        self._check("semmoe_coact_hist", self.lib.semmoe_coact_hist(
            C.byref(c), _stream(), _ptr(topk_ids), int(T_batch), _ptr(load), _ptr(coact)))

    def token_expert_hist(self, token_key, topk_ids, T_batch, V, table):
        c = self._cfg()
        self._check("semmoe_token_expert_hist", self.lib.semmoe_token_expert_hist(
            C.byref(c), _stream(), _ptr(token_key), _ptr(topk_ids), int(T_batch), int(V), _ptr(table)))

    def lookup_tables(self, table_u32, expert_to_rank):
        """host call: numpy uint32 [V,E] and int32 [E] in, three numpy int32 [V] arrays out"""
        import numpy as np
        table_u32 = np.ascontiguousarray(table_u32, dtype=np.uint32)
        e2r = np.ascontiguousarray(expert_to_rank, dtype=np.int32)
        V = table_u32.shape[0]
        dev, conf, level = (np.zeros(V, dtype=np.int32) for _ in range(3))
        c = self._cfg()
        self._check("semmoe_lookup_tables", self.lib.semmoe_lookup_tables(
            C.byref(c), _ptr(table_u32), _ptr(e2r), int(V), _ptr(dev), _ptr(conf), _ptr(level)))
        return dev, conf, level

    def place(self, load_u64, coact_u64, alpha=1, gamma=0, ft_passes=8):
        """host call: numpy uint64 in, three numpy int32 arrays out"""
        import numpy as np
        load_u64 = np.ascontiguousarray(load_u64, dtype=np.uint64)
        coact_u64 = np.ascontiguousarray(coact_u64, dtype=np.uint64)
        E = self.cfg.E
        e2r, phys, inv = (np.zeros(E, dtype=np.int32) for _ in range(3))
        c = self._cfg()
        self._check("semmoe_place", self.lib.semmoe_place(
            C.byref(c), _ptr(load_u64), _ptr(coact_u64), int(alpha), int(gamma), int(ft_passes), _ptr(e2r),
            _ptr(phys), _ptr(inv)))
        return e2r, phys, inv

    def coschedule(self, load_u64, coact_u64, unit_act_u64, unit_len_u64, alpha_e=1, beta_e=1, gamma_e=0, alpha_r=0,
                   beta_r=1, ft_passes=8, n_steps=4, w_load=1, w_comm=1):
        """host call: numpy uint64 in; (expert_to_rank, phys_of_expert, expert_of_phys, unit_rank, step_score,
        best_step) out"""
        import numpy as np
        load_u64 = np.ascontiguousarray(load_u64, dtype=np.uint64)
        coact_u64 = np.ascontiguousarray(coact_u64, dtype=np.uint64)
        unit_act_u64 = np.ascontiguousarray(unit_act_u64, dtype=np.uint64)
        unit_len_u64 = np.ascontiguousarray(unit_len_u64, dtype=np.uint64)
        E = self.cfg.E
        U = unit_len_u64.shape[0]
        if unit_act_u64.shape != (U, E) or load_u64.shape != (E,) or coact_u64.shape != (E, E):
            raise SemMoEError("coschedule: shapes must be load[E], coact[E,E], unit_act[U,E], unit_len[U]", -2)
        e2r, phys, inv = (np.zeros(E, dtype=np.int32) for _ in range(3))
        unit_rank = np.zeros(max(U, 1), dtype=np.int32)
        step_score = np.zeros(max(int(n_steps), 1), dtype=np.int64)
        best = C.c_int32(-1)
        prm = CoschedParams(int(alpha_e), int(beta_e), int(gamma_e), int(alpha_r), int(beta_r), int(w_load),
                            int(w_comm), int(ft_passes), int(n_steps))
        c = self._cfg()
        self._check("semmoe_coschedule", self.lib.semmoe_coschedule(
            C.byref(c), _ptr(load_u64), _ptr(coact_u64), _ptr(unit_act_u64), _ptr(unit_len_u64), int(U),
            C.cast(C.byref(prm), C.c_void_p), _ptr(e2r), _ptr(phys), _ptr(inv), _ptr(unit_rank), _ptr(step_score),
            C.cast(C.byref(best), C.c_void_p)))
        return e2r, phys, inv, unit_rank[:U], step_score, int(best.value)

    def token_labels(self, req_offsets, token_key, req_rank, V):
        """host call: numpy int32 in, three numpy int32 [V] arrays out"""
        import numpy as np
        req_offsets = np.ascontiguousarray(req_offsets, dtype=np.int32)
        token_key = np.ascontiguousarray(token_key, dtype=np.int32)
        req_rank = np.ascontiguousarray(req_rank, dtype=np.int32)
        n_req = req_offsets.shape[0] - 1
        if n_req < 0 or req_rank.shape[0] != n_req or token_key.shape[0] < int(req_offsets[-1]):
            raise SemMoEError("token_labels: req_offsets[n_req+1], req_rank[n_req], token_key[req_offsets[-1]]", -2)
        dev, conf, level = (np.zeros(max(int(V), 1), dtype=np.int32) for _ in range(3))
        c = self._cfg()
        self._check("semmoe_token_labels", self.lib.semmoe_token_labels(
            C.byref(c), _ptr(req_offsets), int(n_req), _ptr(token_key), _ptr(req_rank), int(V), _ptr(dev), _ptr(conf),
            _ptr(level)))
        return dev, conf, level

    def reshuffle(self, topk_ids, expert_to_rank, token_rank, shf, inv_shf, rank_count, cap=None):
        c = self._cfg(**({"cap": cap} if cap is not None else {}))
        self._check("semmoe_reshuffle", self.lib.semmoe_reshuffle(
            C.byref(c), _stream(), _ptr(topk_ids), _ptr(expert_to_rank), _ptr(token_rank), _ptr(shf),
            _ptr(inv_shf), _ptr(rank_count), _ptr(self.ws), self.ws_bytes))

    def reshuffle_static(self, topk_ids, expert_to_rank, token_rank, shf, inv_shf, rank_count, cap=None):
        """the reshuffle on the library's own fixed scratch array: no workspace argument, no allocation"""
        c = self._cfg(**({"cap": cap} if cap is not None else {}))
        self._check("semmoe_reshuffle_static", self.lib.semmoe_reshuffle_static(
            C.byref(c), _stream(), _ptr(topk_ids), _ptr(expert_to_rank), _ptr(token_rank), _ptr(shf),
            _ptr(inv_shf), _ptr(rank_count)))

    def reshuffle_rounds(self, topk_ids, expert_to_rank, rounds, token_rank, shf, inv_shf, rank_count, cap=None):
        c = self._cfg(**({"cap": cap} if cap is not None else {}))
        self._check("semmoe_reshuffle_rounds", self.lib.semmoe_reshuffle_rounds(
            C.byref(c), _stream(), _ptr(topk_ids), _ptr(expert_to_rank), int(rounds), _ptr(token_rank), _ptr(shf),
            _ptr(inv_shf), _ptr(rank_count), _ptr(self.ws), self.ws_bytes))

    def reshuffle_refine(self, topk_ids, expert_to_rank, rounds, max_cycles, token_rank, shf, inv_shf, rank_count,
                         info, cap=None):
        c = self._cfg(**({"cap": cap} if cap is not None else {}))
        self._check("semmoe_reshuffle_refine", self.lib.semmoe_reshuffle_refine(
            C.byref(c), _stream(), _ptr(topk_ids), _ptr(expert_to_rank), int(rounds), int(max_cycles),
            _ptr(token_rank), _ptr(shf), _ptr(inv_shf), _ptr(rank_count), _ptr(info), _ptr(self.ws), self.ws_bytes))

    def reshuffle_lookup(self, token_key, V, dev, conf_q16, level, thr_q16, token_rank, shf, inv_shf, rank_count,
                         cap=None):
        c = self._cfg(**({"cap": cap} if cap is not None else {}))
        self._check("semmoe_reshuffle_lookup", self.lib.semmoe_reshuffle_lookup(
            C.byref(c), _stream(), _ptr(token_key), int(V), _ptr(dev), _ptr(conf_q16), _ptr(level), int(thr_q16),
            _ptr(token_rank), _ptr(shf), _ptr(inv_shf), _ptr(rank_count), _ptr(self.ws), self.ws_bytes))

    def reshuffle_cond(self, token_key, V, dev, conf_q16, level, seq_key, VA, dev_a, conf_a_q16, level_a, thr_q16,
                       token_rank, shf, inv_shf, rank_count, cap=None):
        c = self._cfg(**({"cap": cap} if cap is not None else {}))
        self._check("semmoe_reshuffle_cond", self.lib.semmoe_reshuffle_cond(
            C.byref(c), _stream(), _ptr(token_key), int(V), _ptr(dev), _ptr(conf_q16), _ptr(level), _ptr(seq_key),
            int(VA), _ptr(dev_a), _ptr(conf_a_q16), _ptr(level_a), int(thr_q16), _ptr(token_rank), _ptr(shf),
            _ptr(inv_shf), _ptr(rank_count), _ptr(self.ws), self.ws_bytes))

    def device_sequence(self, topk_ids, expert_to_rank, T_batch, seq_in, seq_out):
        c = self._cfg()
        self._check("semmoe_device_sequence", self.lib.semmoe_device_sequence(
            C.byref(c), _stream(), _ptr(topk_ids), _ptr(expert_to_rank), int(T_batch), _ptr(seq_in), _ptr(seq_out)))

    def request_schedule(self, req_offsets, n_req, token_key, V, dev, req_rank, token_rank, shf, inv_shf, rank_count):
        c = self._cfg()
        self._check("semmoe_request_schedule", self.lib.semmoe_request_schedule(
            C.byref(c), _stream(), _ptr(req_offsets), int(n_req), _ptr(token_key), int(V), _ptr(dev), _ptr(req_rank),
            _ptr(token_rank), _ptr(shf), _ptr(inv_shf), _ptr(rank_count), _ptr(self.ws), self.ws_bytes))

    def dispatch(self, X, topk_ids, token_rank, shf, phys_of_expert, X_perm, slot_of_pair, pair_of_slot,
                 expert_offsets, rank_offsets, send_matrix, remote_pairs):
        c = self._cfg()
        self._check("semmoe_dispatch", self.lib.semmoe_dispatch(
            C.byref(c), _stream(), _ptr(X), _ptr(topk_ids), _ptr(token_rank), _ptr(shf), _ptr(phys_of_expert),
            _ptr(X_perm), _ptr(slot_of_pair), _ptr(pair_of_slot), _ptr(expert_offsets), _ptr(rank_offsets),
            _ptr(send_matrix), _ptr(remote_pairs), _ptr(self.ws), self.ws_bytes))

    def dispatch_index(self, topk_ids, token_rank, shf, phys_of_expert, slot_of_pair, pair_of_slot, expert_offsets,
                       rank_offsets, send_matrix, remote_pairs):
        c = self._cfg()
        self._check("semmoe_dispatch_index", self.lib.semmoe_dispatch_index(
            C.byref(c), _stream(), _ptr(topk_ids), _ptr(token_rank), _ptr(shf), _ptr(phys_of_expert),
            _ptr(slot_of_pair), _ptr(pair_of_slot), _ptr(expert_offsets), _ptr(rank_offsets), _ptr(send_matrix),
            _ptr(remote_pairs), _ptr(self.ws), self.ws_bytes))

    def dispatch_rows(self, X, slot_of_pair, X_perm):
        c = self._cfg()
        self._check("semmoe_dispatch_rows", self.lib.semmoe_dispatch_rows(
            C.byref(c), _stream(), _ptr(X), _ptr(slot_of_pair), _ptr(X_perm)))

    def expert_ffn(self, rank, X_perm, expert_offsets, expert_of_phys, W_gu, W_down, Y):
        c = self._cfg()
        self._check("semmoe_expert_ffn", self.lib.semmoe_expert_ffn(
            C.byref(c), _stream(), int(rank), _ptr(X_perm), _ptr(expert_offsets), _ptr(expert_of_phys),
            _ptr(W_gu), _ptr(W_down), _ptr(Y), _ptr(self.ws), self.ws_bytes))

    def shared_ffn(self, X, n_tokens, W_gu_sh, W_down_sh, Y_shared):
        """the shared expert has a workspace of its own (n_tokens x F activations), so that it may run on another
        stream beside the routed path's calls, which share `self.ws`"""
        c = self._cfg()
        need = int(n_tokens) * self.cfg.F * (2 if self.cfg.dtype == BF16 else 4) + 512
        if self.ws_shared is None or self.ws_shared.numel() < need:
            import torch
            self.ws_shared = torch.empty(need, dtype=torch.uint8, device=X.device)
        self._check("semmoe_shared_ffn", self.lib.semmoe_shared_ffn(
            C.byref(c), _stream(), _ptr(X), int(n_tokens), _ptr(W_gu_sh), _ptr(W_down_sh), _ptr(Y_shared),
            _ptr(self.ws_shared), self.ws_shared.numel()))

    def probe_copy(self, dst, src, nbytes):
        self._check("semmoe_probe_copy", self.lib.semmoe_probe_copy(_stream(), _ptr(dst), _ptr(src), int(nbytes)))

    def probe_stream(self, buf, nbytes, write, sink):
        self._check("semmoe_probe_stream", self.lib.semmoe_probe_stream(_stream(), _ptr(buf), int(nbytes), int(bool(write)),
                                                                        _ptr(sink)))

    def probe_mfma(self, operands, iters, sink):
        """returns the flops of the launch"""
        fl = C.c_double(0.0)
        self._check("semmoe_probe_mfma", self.lib.semmoe_probe_mfma(_stream(), _ptr(operands), int(iters), _ptr(sink),
                                                                    C.byref(fl)))
        return fl.value

    def probe_tile_loop(self, panels, n_panels, row_bytes, variant, n_slices, sink):
        """returns the flops of the launch"""
        fl = C.c_double(0.0)
        self._check("semmoe_probe_tile_loop", self.lib.semmoe_probe_tile_loop(
            _stream(), _ptr(panels), int(n_panels), int(row_bytes), int(variant), int(n_slices), _ptr(sink), C.byref(fl)))
        return fl.value

    def combine(self, Y, slot_of_pair, topk_w, Out, Y_shared=None):
        c = self._cfg()
        self._check("semmoe_combine", self.lib.semmoe_combine(
            C.byref(c), _stream(), _ptr(Y), _ptr(slot_of_pair), _ptr(topk_w), _ptr(Y_shared), _ptr(Out)))
