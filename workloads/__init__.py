"""Seeded synthetic inputs for the semantic-parallel MoE layer.

This module only draws numbers and shapes: hidden states, router and expert
weights, latent token classes and the per-class logit bias that makes routing
"semantic" (a token's experts concentrate on a small static subset, the
behaviour the paper reports in Sec. 3.2 / Table 1).  It holds none of the
method's arithmetic (no routing, placement, sorting, FFN or combine), so the
CPU oracle and the HIP library can both be fed from it without sharing code.

Every tensor has its own counter-based stream (Philox keyed by
(seed, stream id, sub id)), so any single expert's weights can be drawn
without drawing the others.

Arrays are float32.  For the bf16 workloads every value is already rounded to
the nearest bf16 (ties to even), so both sides read identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Tuple

import numpy as np

# stream ids (one per tensor kind)
_S_X, _S_WR, _S_PERM, _S_CLASS, _S_BIAS, _S_WGU, _S_WDOWN, _S_FREE, _S_SH, _S_KEY, _S_REQ, _S_SHARED = range(12)
PROFILE_SEED_OFFSET = 1000


@dataclass(frozen=True)
class Workload:
    name: str
    T: int            # tokens in the measured batch
    d: int            # hidden width
    E: int            # routed experts
    k: int            # experts per token
    F: int            # expert FFN width
    D: int            # logical expert-parallel ranks
    dtype: str        # "fp32" | "bf16"
    score: str        # "softmax" | "sigmoid"
    renorm: bool
    C: int            # latent semantic classes
    bias_lo: float    # per-class logit bias on the class's expert cluster
    bias_hi: float    # (bias_lo == bias_hi: constant bias)
    class_mix: str    # "uniform" | "zipf"
    zipf_s: float = 1.1
    free_frac: float = 0.0      # share of class-free tokens (token_class = -1)
    n_group: int = 1
    topk_group: int = 1
    routed_scale: float = 1.0
    n_shared: int = 0
    T_profile: int = 0          # tokens of the profiling batch (0: same as T)
    seed: int = 0
    weight_std: float = 0.02

    @property
    def m(self) -> int:
        """experts per rank (also the size of a class's expert cluster)"""
        return self.E // self.D

    @property
    def P(self) -> int:
        return self.T * self.k

    @property
    def cap(self) -> int:
        """tokens per rank at capacity factor 1"""
        return -(-self.T // self.D)

    @property
    def profile_tokens(self) -> int:
        return self.T_profile or self.T

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


CONFIGS: Dict[str, Workload] = {
    # configs[0]: tiny fp32 layer
    "c1_tiny_fp32": Workload("c1_tiny_fp32", T=256, d=512, E=16, k=2, F=1024, D=4, dtype="fp32",
                             score="softmax", renorm=False, C=4, bias_lo=2.0, bias_hi=2.0,
                             class_mix="uniform"),
    # configs[1]: Qwen3-30B-A3B-shaped layer
    "c2_qwen3_30b": Workload("c2_qwen3_30b", T=8192, d=2048, E=128, k=8, F=768, D=8, dtype="bf16",
                             score="softmax", renorm=True, C=16, bias_lo=1.5, bias_hi=1.5,
                             class_mix="zipf", zipf_s=1.1),
    # configs[2]: DeepSeek-V3-shaped layer (the largest of the five; it fits one GPU)
    "c3_deepseek_v3": Workload("c3_deepseek_v3", T=16384, d=7168, E=256, k=8, F=2048, D=32, dtype="bf16",
                               score="sigmoid", renorm=True, C=32, bias_lo=1.5, bias_hi=1.5,
                               class_mix="uniform", n_group=8, topk_group=4, n_shared=1),
    # configs[3]: GPT-OSS-120B-shaped layer
    "c4_gpt_oss_120b": Workload("c4_gpt_oss_120b", T=32768, d=2880, E=128, k=4, F=2880, D=16, dtype="bf16",
                                score="softmax", renorm=True, C=32, bias_lo=0.5, bias_hi=2.5,
                                class_mix="uniform", free_frac=0.10),
    # configs[4]: decode-shaped Qwen3-235B-A22B layer
    "c5_qwen3_235b_decode": Workload("c5_qwen3_235b_decode", T=256, d=4096, E=128, k=8, F=1536, D=8,
                                     dtype="bf16", score="softmax", renorm=True, C=16, bias_lo=1.5,
                                     bias_hi=1.5, class_mix="uniform", T_profile=65536),
}
CONFIG_ORDER = list(CONFIGS)


def small(name: str = "s_bf16", **kw) -> Workload:
    """A small workload for tests: spans several tiles and ragged tails."""
    base = dict(name=name, T=200, d=64, E=16, k=2, F=96, D=4, dtype="bf16", score="softmax", renorm=True,
                C=4, bias_lo=1.5, bias_hi=1.5, class_mix="uniform")
    base.update(kw)
    return Workload(**base)


# ----------------------------------------------------------------------------- bf16 helpers (format only)
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bf16 (ties to even), returned as float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------- generators
def _rng(w: Workload, stream: int, sub: int = 0, profile: bool = False) -> np.random.Generator:
    seed = w.seed + (PROFILE_SEED_OFFSET if profile else 0)
    return np.random.Generator(np.random.Philox(key=[(seed << 32) | (stream << 24) | sub, 0x5E77_0E00]))


def _normal(w: Workload, rng: np.random.Generator, shape, std: float) -> np.ndarray:
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if w.dtype == "bf16":
        a = round_to_bf16(a)
    return a


def hidden(w: Workload, profile: bool = False, n: Optional[int] = None) -> np.ndarray:
    """X[T,d] ~ N(0,1)"""
    n = n if n is not None else (w.profile_tokens if profile else w.T)
    return _normal(w, _rng(w, _S_X, 0, profile), (n, w.d), 1.0)


def router_weight(w: Workload, layer: int = 0) -> np.ndarray:
    """W_r[E,d] ~ N(0, 0.02): one row per expert (the paper's gate-matrix column).  layer 0 is the layer the path
    runs; layer 1, 2, ... are the MoE layers before it (their own weights, scramble and clusters), used only to
    give tokens a routing history for the inter-layer table."""
    return _normal(w, _rng(w, _S_WR, layer), (w.E, w.d), w.weight_std)


def expert_scramble(w: Workload, layer: int = 0) -> np.ndarray:
    """Seeded permutation pi of expert ids, so that contiguous (vanilla) placement does not
    already match the semantic clusters."""
    return _rng(w, _S_PERM, layer).permutation(w.E).astype(np.int32)


def class_clusters(w: Workload, layer: int = 0) -> np.ndarray:
    """cluster[c, j] = pi[(c * E/C + j) mod E], j < m.  Disjoint when E/C == m, overlapping otherwise."""
    pi = expert_scramble(w, layer)
    stride = max(w.E // w.C, 1)
    idx = (np.arange(w.C)[:, None] * stride + np.arange(w.m)[None, :]) % w.E
    return pi[idx]


def class_bias(w: Workload, layer: int = 0) -> np.ndarray:
    """class_bias[C,E] fp32: beta_c on the class's cluster, 0 elsewhere."""
    cl = class_clusters(w, layer)
    if w.bias_lo == w.bias_hi:
        beta = np.full(w.C, w.bias_lo, dtype=np.float32)
    else:
        beta = _rng(w, _S_BIAS, layer).uniform(w.bias_lo, w.bias_hi, size=w.C).astype(np.float32)
    b = np.zeros((w.C, w.E), dtype=np.float32)
    for c in range(w.C):
        b[c, cl[c]] = beta[c]
    return b


def token_class(w: Workload, profile: bool = False, n: Optional[int] = None) -> np.ndarray:
    """token_class[T] int32 in [0,C), or -1 for class-free tokens."""
    n = n if n is not None else (w.profile_tokens if profile else w.T)
    rng = _rng(w, _S_CLASS, 0, profile)
    if w.class_mix == "zipf":
        p = (np.arange(w.C) + 1.0) ** (-w.zipf_s)
        p /= p.sum()
        cls = rng.choice(w.C, size=n, p=p)
    else:
        cls = rng.integers(0, w.C, size=n)
    cls = cls.astype(np.int32)
    if w.free_frac > 0:
        free = _rng(w, _S_FREE, 0, profile).random(n) < w.free_frac
        cls[free] = -1
    return cls


KEYS_PER_CLASS = 64


def vocab_size(w: Workload, shared: bool = False) -> int:
    """size of the synthetic vocabulary: KEYS_PER_CLASS keys per latent class + as many class-free keys
    (+ as many keys shared by all classes when `shared`)"""
    return (w.C + 1 + (1 if shared else 0)) * KEYS_PER_CLASS


def token_key(w: Workload, profile: bool = False, n: Optional[int] = None, shared_frac: float = 0.0) -> np.ndarray:
    """token_key[T] int32 in [0, vocab_size): a synthetic token id.  Every class owns KEYS_PER_CLASS keys
    (the tokens of a class are uniform over them); class-free tokens draw from the next KEYS_PER_CLASS keys.
    Stands in for the vocabulary ids the paper's lookup tables are indexed by.
    shared_frac > 0: that share of the tokens, of whatever class, carries one of KEYS_PER_CLASS further keys that all
    classes share (ids from vocab_size(w) on; the vocabulary is then vocab_size(w, shared=True)): token ids whose
    routing depends on the context and not on the id, which is what the inter-layer table is there for."""
    cls = token_class(w, profile, n)
    sub = _rng(w, _S_KEY, 0, profile).integers(0, KEYS_PER_CLASS, size=cls.shape[0])
    base = np.where(cls >= 0, cls, w.C).astype(np.int64) * KEYS_PER_CLASS
    if shared_frac > 0:
        amb = _rng(w, _S_SHARED, 0, profile).random(cls.shape[0]) < shared_frac
        base[amb] = (w.C + 1) * KEYS_PER_CLASS
    return (base + sub).astype(np.int32)


def requests(w: Workload, profile: bool = False, n: Optional[int] = None, min_len: int = 16, max_len: int = 1024,
             topic_frac: float = 0.8) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Synthetic requests for the request-level (Attention-DP) scenario: the batch of n tokens is cut into runs,
    one per request, with lengths log-uniform in [min_len, max_len] (the last one truncated to fit).  A request
    has a topic class drawn from the workload's class mix; each of its tokens carries the topic with probability
    topic_frac, otherwise it is an ordinary token of the batch mix (`token_class`).  Keys follow the classes as in
    `token_key`.  Returns (req_offsets[n_req+1] int32, token_class[n] int32, token_key[n] int32)."""
    n = n if n is not None else (w.profile_tokens if profile else w.T)
    rng = _rng(w, _S_REQ, 0, profile)
    lens = []
    left = n
    while left > 0:
        ln = int(np.exp(rng.uniform(np.log(min_len), np.log(max_len))))
        ln = max(1, min(ln, left))
        lens.append(ln)
        left -= ln
    off = np.zeros(len(lens) + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    if w.class_mix == "zipf":
        p = (np.arange(w.C) + 1.0) ** (-w.zipf_s)
        p /= p.sum()
        topic = rng.choice(w.C, size=len(lens), p=p)
    else:
        topic = rng.integers(0, w.C, size=len(lens))
    cls = token_class(w, profile, n).copy()
    on_topic = rng.random(n) < topic_frac
    req_of = np.repeat(np.arange(len(lens)), lens)
    cls[on_topic] = topic[req_of[on_topic]].astype(np.int32)
    sub = _rng(w, _S_REQ, 1, profile).integers(0, KEYS_PER_CLASS, size=n)
    base = np.where(cls >= 0, cls, w.C).astype(np.int64) * KEYS_PER_CLASS
    return off, cls, (base + sub).astype(np.int32)


def expert_weight(w: Workload, e: int) -> Tuple[np.ndarray, np.ndarray]:
    """(W_gu[e] [2F,d] = [gate rows; up rows], W_down[e] [d,F]) ~ N(0, 0.02)"""
    wgu = _normal(w, _rng(w, _S_WGU, e + 1), (2 * w.F, w.d), w.weight_std)
    wdn = _normal(w, _rng(w, _S_WDOWN, e + 1), (w.d, w.F), w.weight_std)
    return wgu, wdn


def shared_weight(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """weights of the shared expert (same shapes as a routed expert)"""
    wgu = _normal(w, _rng(w, _S_SH, 1), (2 * w.F, w.d), w.weight_std)
    wdn = _normal(w, _rng(w, _S_SH, 2), (w.d, w.F), w.weight_std)
    return wgu, wdn


def all_expert_weights(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """W_gu[E,2F,d], W_down[E,d,F] (only for workloads whose experts fit host memory)"""
    wgu = np.empty((w.E, 2 * w.F, w.d), dtype=np.float32)
    wdn = np.empty((w.E, w.d, w.F), dtype=np.float32)
    for e in range(w.E):
        wgu[e], wdn[e] = expert_weight(w, e)
    return wgu, wdn


def uniform_random_ids(T: int, E: int, k: int, seed: int = 0) -> np.ndarray:
    """class-free routing: k distinct experts per token, uniform (for the LAR = 1/D pin)."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0xA11CE]))
    r = rng.random((T, E))
    return np.argsort(r, axis=1, kind="stable")[:, :k].astype(np.int32)
