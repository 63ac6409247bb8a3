"""The allocation-free reshuffle (`semmoe_reshuffle_static`: scratch in a fixed array of the library's code
object) against `semmoe_reshuffle` (scratch in the caller's workspace), through the C ABI: two calls in a row on
the same GPU, the second on a smaller batch, every output bit for bit, and against the oracle."""
import numpy as np
import pytest
import torch

import workloads as WL
from oracle import semmoe_oracle as O
import paper_2503_04398_amd as S
from tests import harness as H

pytestmark = pytest.mark.gpu


def _planted_ids(T, E, D, k, seed):
    """clustered routing so that capacity binds: a token's experts mostly lie on one rank"""
    r = np.random.default_rng(seed)
    m = E // D
    cls = r.integers(0, D, size=T) * (r.random(T) < 0.7) + (r.random(T) >= 0.7) * 0     # rank 0 is over-subscribed
    score = r.random((T, E)) + 0.6 * ((np.arange(E)[None, :] // m) == cls[:, None])
    return np.argsort(-score, axis=1, kind="stable")[:, :k].astype(np.int32)


def _both(T, E, D, k, seed):
    w = WL.small(T=T, E=E, D=D, k=k)
    ids = _planted_ids(T, E, D, k, seed)
    e2r = (np.arange(E) // (E // D)).astype(np.int32)
    out = {}
    for which in ("workspace", "static"):
        lay = H.Layer(w)
        lay.set_routing(ids)
        lay.e2r = H.to_dev(e2r)
        for t in (lay.token_rank, lay.shf, lay.inv_shf, lay.rank_count):
            t.fill_(-7)
        if which == "workspace":
            lay.m.reshuffle(lay.ids, lay.e2r, lay.token_rank, lay.shf, lay.inv_shf, lay.rank_count)
        else:
            lay.m.reshuffle_static(lay.ids, lay.e2r, lay.token_rank, lay.shf, lay.inv_shf, lay.rank_count)
        torch.cuda.synchronize()
        out[which] = tuple(H.to_np(t) for t in (lay.token_rank, lay.shf, lay.inv_shf, lay.rank_count))
    want = O.reshuffle(ids, e2r, D, w.cap)
    return out, want


def test_reshuffle_static_equals_reshuffle_on_two_calls_in_a_row():
    # 40000 and 5000 tokens: both above the single-workgroup limit, so both calls run the kernels that use the
    # scratch (per-token words and per-block count tables); the second call finds the first call's contents there
    for T, E, D, k, seed in ((40000, 64, 16, 4, 1), (5000, 32, 8, 2, 2)):
        print("reshuffle_static", dict(T=T, E=E, D=D, k=k), flush=True)
        out, want = _both(T, E, D, k, seed)
        for a, b, x, nm in zip(out["static"], out["workspace"], want, ("token_rank", "shf", "inv_shf", "rank_count")):
            assert (a == b).all(), nm
            assert (a == x).all(), nm + " vs oracle"
        assert out["static"][3].max() == -(-T // D)          # capacity binds in this input
