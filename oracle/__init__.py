"""CPU oracle (test infrastructure only).

Thin ctypes loader for ``tg_oracle.c``: exact brute-force k-NN (O-BF) and the
two-phase NN-Descent of Algorithm 1 (O-NND), both single-threaded and in
double precision; and for ``tg_prune_oracle.c``: the rank-based pruning of a
k-NN graph by detourable routes; and for ``tg_filter_oracle.c``: the distance-based
(NSG / Vamana) pruning over 1-hop or 2-hop candidates; and for ``tg_merge_oracle.c``: the merge of
a local index into the global one.  Nothing in the product path may import this package; it is
for ``tests/``, the smoke check and the benchmark's CPU-baseline leg.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tg_oracle.c")
_SRC2 = os.path.join(_HERE, "tg_prune_oracle.c")
_SRC3 = os.path.join(_HERE, "tg_filter_oracle.c")
_SRC4 = os.path.join(_HERE, "tg_merge_oracle.c")
_LIB = os.path.join(_HERE, "libtg_oracle.so")

METRIC_L2, METRIC_IP, METRIC_COSINE = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, no HIP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(s) for s in (_SRC, _SRC2, _SRC3, _SRC4)):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-o", tmp, _SRC, _SRC2, _SRC3, _SRC4, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, i32, u64, dbl, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_uint64, ctypes.c_double, ctypes.c_void_p
        L.oracle_mix64.restype = u64
        L.oracle_mix64.argtypes = [u64]
        L.oracle_hash3.restype = u64
        L.oracle_hash3.argtypes = [u64, u64, u64, u64]
        L.oracle_slot_of.restype = ctypes.c_uint32
        L.oracle_slot_of.argtypes = [u64, i32, i32, i32, i32, i32]
        L.oracle_distance.restype = dbl
        L.oracle_distance.argtypes = [vp, i64, i32, i64, i64]
        L.obf_knn.restype = i32
        L.obf_knn.argtypes = [vp, i64, i64, i32, i32, vp, i64, vp, vp]
        L.onnd_create.restype = vp
        L.onnd_create.argtypes = [vp, i64, i64, i32, i32] + [i32] * 12 + [u64]
        L.onnd_destroy.argtypes = [vp]
        L.onnd_export.argtypes = [vp, vp, vp, vp]
        L.onnd_counters.argtypes = [vp, vp]
        L.onnd_import.argtypes = [vp, vp, vp, vp]
        L.onnd_init.argtypes = [vp]
        L.onnd_phase1_sample.argtypes = [vp]
        L.onnd_block.argtypes = [vp, i64, vp, vp]
        L.oprune_rank.restype = i32
        L.oprune_rank.argtypes = [vp, i64, i64, i32, i32, vp, vp]
        L.ofilter_dist.restype = i32
        L.ofilter_dist.argtypes = [vp, i64, i32, vp, i32, i64, i32, i32, ctypes.c_float, i32, vp, vp, vp]
        L.oangle_at_many.restype = None
        L.oangle_at_many.argtypes = [vp, vp, vp, vp, i64]
        L.ofilter.restype = i32
        L.ofilter.argtypes = [vp, i64, i32, vp, i32, i64, i32, i32, i32, ctypes.c_float, i32, vp, vp, vp]
        L.omerge_local.restype = i32
        L.omerge_local.argtypes = [vp, vp, i64, i32, vp, vp, i64, i32, vp]
        L.oracle_merge_list.restype = i64
        L.oracle_merge_list.argtypes = [i32, i64, vp, vp, vp, vp, vp, i64]
        L.onnd_phase1_round.restype = i64
        L.onnd_phase1_round.argtypes = [vp]
        L.onnd_begin_phase2.argtypes = [vp]
        L.onnd_phase2_round.restype = i64
        L.onnd_phase2_round.argtypes = [vp]
        L.onnd_run.argtypes = [vp, i32, i32, dbl, vp]
        L.oracle_recall.restype = dbl
        L.oracle_recall.argtypes = [vp, vp, i64, i32]
        _lib = L
    return _lib


def _f32(X):
    X = np.ascontiguousarray(X, dtype=np.float32)
    assert X.ndim == 2
    return X


def mix64(z: int) -> int:
    return lib().oracle_mix64(z & (2**64 - 1))


def hash3(seed: int, tag: int, x: int, y: int) -> int:
    return lib().oracle_hash3(seed, tag, x, y)


def slot_of(seed: int, round_: int, t: int, v: int, g: int, C: int) -> int:
    """Slot (of target t's C) that takes the candidate anchor v's block found in opponent group g."""
    return lib().oracle_slot_of(seed, round_, t, v, g, C)


def distance(X, metric: int, a: int, b: int) -> float:
    X = _f32(X)
    return lib().oracle_distance(X.ctypes.data, X.shape[1], metric, a, b)


def brute_force_knn(X, k: int, metric: int = METRIC_L2, rows=None):
    """O-BF: exact k-NN of the given rows (all rows if None) under (dist, id) order."""
    X = _f32(X)
    n, d = X.shape
    if rows is None:
        rows_arr, nq, rp = None, n, None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        nq, rp = len(rows_arr), rows_arr.ctypes.data
    ids = np.empty((nq, k), dtype=np.int32)
    dist = np.empty((nq, k), dtype=np.float64)
    rc = lib().obf_knn(X.ctypes.data, n, d, k, metric, rp, nq, ids.ctypes.data, dist.ctypes.data)
    if rc != 0:
        raise ValueError("obf_knn: invalid arguments")
    return ids, dist


def recall(ids, truth) -> float:
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    truth = np.ascontiguousarray(truth, dtype=np.int32)
    assert ids.shape == truth.shape
    return lib().oracle_recall(ids.ctypes.data, truth.ctypes.data, ids.shape[0], ids.shape[1])


def merge_list(self_id, ids, dist, fresh, cand_ids, cand_dist):
    """The neighbour-list update rule on explicit arrays; returns (ids, dist, fresh, inserted)."""
    ids = np.array(ids, dtype=np.int32)
    dist = np.array(dist, dtype=np.float64)
    fresh = np.array(fresh, dtype=np.uint8)
    cid = np.ascontiguousarray(cand_ids, dtype=np.int32)
    cd = np.ascontiguousarray(cand_dist, dtype=np.float64)
    ins = lib().oracle_merge_list(len(ids), self_id, ids.ctypes.data, dist.ctypes.data, fresh.ctypes.data,
                                  cid.ctypes.data, cd.ctypes.data, len(cid))
    return ids, dist, fresh, ins


def prune_rank(ids, d_out: int, n_do=None):
    """Rank-based pruning (sections 3.2 and 5.2) of the rows of the first n_do nodes (default: all):
    returns (out_ids n_do x d_out, counts n_do x k)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    n, k = ids.shape
    n_do = n if n_do is None else int(n_do)
    out = np.empty((n_do, d_out), dtype=np.int32)
    cnt = np.empty((n_do, k), dtype=np.int32)
    rc = lib().oprune_rank(ids.ctypes.data, n, n_do, k, d_out, out.ctypes.data, cnt.ctypes.data)
    if rc != 0:
        raise ValueError("bad arguments")
    return out, cnt


def filter_dist(X, ids, hops: int, cand_size: int, alpha: float, d_out: int, n_do=None):
    """Distance-based pruning (section 3.2: NSG for alpha = 1, Vamana for alpha > 1) over the 1-hop or
    2-hop candidates of the graph ``ids`` (section 5.1), squared L2.  Returns (out_ids n_do x d_out
    padded with -1, degrees, margins): see tg_filter_oracle.c for the margin."""
    X = _f32(X)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    n, k = ids.shape
    assert X.shape[0] == n
    n_do = n if n_do is None else int(n_do)
    out = np.empty((n_do, d_out), dtype=np.int32)
    deg = np.empty(n_do, dtype=np.int32)
    margin = np.empty(n_do, dtype=np.float64)
    rc = lib().ofilter_dist(X.ctypes.data, n, X.shape[1], ids.ctypes.data, k, n_do, hops, cand_size,
                            float(alpha), d_out, out.ctypes.data, deg.ctypes.data, margin.ctypes.data)
    if rc != 0:
        raise ValueError("bad arguments")
    return out, deg, margin


def filter_angle(X, ids, hops: int, cand_size: int, gamma_deg: float, d_out: int, n_do=None):
    """Angle-based pruning (section 3.2, the NSSG rule: a candidate is inserted iff its direction from p makes
    an angle above gamma with that of every neighbour inserted before) over the 1-hop or 2-hop candidates.
    Returns (out_ids n_do x d_out padded with -1, degrees, margins)."""
    X = _f32(X)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    n, k = ids.shape
    assert X.shape[0] == n
    n_do = n if n_do is None else int(n_do)
    out = np.empty((n_do, d_out), dtype=np.int32)
    deg = np.empty(n_do, dtype=np.int32)
    margin = np.empty(n_do, dtype=np.float64)
    rc = lib().ofilter(X.ctypes.data, n, X.shape[1], ids.ctypes.data, k, n_do, hops, cand_size, 1, float(gamma_deg), d_out,
                       out.ctypes.data, deg.ctypes.data, margin.ctypes.data)
    if rc != 0:
        raise ValueError("bad arguments")
    return out, deg, margin


def filter_dpg(X, ids, hops: int, cand_size: int, d_out: int, n_do=None):
    """Dispersion pruning (section 3.2, the DPG rule: greedy insertion of the candidate whose angles to the inserted
    nodes add up to the most) over the 1-hop or 2-hop candidates.  Returns (out_ids in insertion order padded with
    -1, degrees, margins in radians)."""
    X = _f32(X)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    n, k = ids.shape
    assert X.shape[0] == n
    n_do = n if n_do is None else int(n_do)
    out = np.empty((n_do, d_out), dtype=np.int32)
    deg = np.empty(n_do, dtype=np.int32)
    margin = np.empty(n_do, dtype=np.float64)
    rc = lib().ofilter(X.ctypes.data, n, X.shape[1], ids.ctypes.data, k, n_do, hops, cand_size, 2, 0.0, d_out,
                       out.ctypes.data, deg.ctypes.data, margin.ctypes.data)
    if rc != 0:
        raise ValueError("bad arguments")
    return out, deg, margin


def angle_at(a, b, c):
    """The angle (radians, float32) at p between p -> r and p -> c from the squared lengths |p r|^2, |p c|^2, |r c|^2,
    elementwise, as the dispersion rule computes it."""
    a, b, c = (np.ascontiguousarray(v, dtype=np.float32).ravel() for v in (a, b, c))
    assert a.size == b.size == c.size
    out = np.empty(a.shape, dtype=np.float32)
    lib().oangle_at_many(a.ctypes.data, b.ctypes.data, c.ctypes.data, out.ctypes.data, a.size)
    return out


def merge_local(g_ids, g_dist, l_ids, l_dist, l2g):
    """Merges a local index (local numbering, ``l2g`` gives the global ids) into the global lists
    (section 6.1), in place: every touched row becomes the k closest of the union."""
    assert g_ids.dtype == np.int32 and g_dist.dtype == np.float32 and g_ids.flags.c_contiguous and g_dist.flags.c_contiguous
    l_ids = np.ascontiguousarray(l_ids, dtype=np.int32)
    l_dist = np.ascontiguousarray(l_dist, dtype=np.float32)
    l2g = np.ascontiguousarray(l2g, dtype=np.int32)
    n, k = g_ids.shape
    nl, kl = l_ids.shape
    rc = lib().omerge_local(g_ids.ctypes.data, g_dist.ctypes.data, n, k, l_ids.ctypes.data, l_dist.ctypes.data, nl, kl,
                            l2g.ctypes.data)
    if rc != 0:
        raise ValueError("bad arguments")


# The bounded hand-over of candidates that the HIP library's local join uses (include/tagore_knn.h, parameters
# C and parts): per member and group of eight consecutive block positions the closest candidate that the
# member's list does not hold yet.  A test that follows a device build step by step passes these, with the
# build's C and parts; the reference mode of O-NND (the defaults of NNDescent) has none of it.
DEVICE_HANDOVER = dict(retain=1, tile=8, ng_row=8, ng_col=8, exclude_listed=True)


def device_model(prm):
    """Keyword arguments of NNDescent that follow a build with the parameters ``prm`` (a tg_knn_params) step by step."""
    return dict(S=prm.S, R=prm.R, C=prm.C, parts=prm.parts, m=prm.m, seed=prm.seed, **DEVICE_HANDOVER)


class NNDescent:
    """O-NND: one object per build; methods are the steps of Algorithm 1.

    The defaults are the plain method (every evaluated pair offered to both nodes, unbounded candidate
    lists, one update per round).  ``retain``, ``tile``, ``ng_row``, ``ng_col``, ``C``, ``exclude_listed``
    and ``parts`` model a bounded hand-over of candidates (see tg_oracle.c) and are set by the tests that
    follow a device build step by step."""

    def __init__(self, X, k, metric=METRIC_L2, S=None, R=None, C=0, retain=0, tile=16,
                 ng_row=2, ng_col=2, m=2, all_block=False, use_threshold=True, seed=1,
                 exclude_listed=False, parts=1):
        self.X = _f32(X)
        self.n, self.d = self.X.shape
        self.k = k
        S = min(k, 32) if S is None else S
        R = 32 if R is None else R
        self.S, self.R = S, R
        self._h = lib().onnd_create(self.X.ctypes.data, self.n, self.d, k, metric, S, R, C,
                                    retain, tile, ng_row, ng_col, m, int(all_block),
                                    int(use_threshold), int(exclude_listed), int(parts), seed)
        if not self._h:
            raise ValueError("onnd_create: invalid arguments")

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.onnd_destroy(self._h)
            self._h = None

    def init(self):
        lib().onnd_init(self._h)

    def phase1_sample(self):
        """Draw this round's forward and reverse samples without running the round."""
        lib().onnd_phase1_sample(self._h)

    def block(self, v: int):
        """(NEW ids, OLD ids) of anchor v for the samples last drawn."""
        blk = np.empty(2 * self.S + 2 * self.R, dtype=np.int32)
        sizes = (ctypes.c_int * 2)()
        lib().onnd_block(self._h, v, blk.ctypes.data, sizes)
        return blk[:sizes[0]].copy(), blk[sizes[0]:sizes[0] + sizes[1]].copy()

    def phase1_round(self) -> int:
        return lib().onnd_phase1_round(self._h)

    def begin_phase2(self):
        lib().onnd_begin_phase2(self._h)

    def phase2_round(self) -> int:
        return lib().onnd_phase2_round(self._h)

    def run(self, it1, it2, delta=0.0):
        done = (ctypes.c_int * 2)()
        lib().onnd_run(self._h, it1, it2, delta, done)
        return done[0], done[1]

    def set_graph(self, ids, dist, fresh):
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        dist = np.ascontiguousarray(dist, dtype=np.float64)
        fresh = np.ascontiguousarray(fresh, dtype=np.uint8)
        assert ids.shape == dist.shape == fresh.shape == (self.n, self.k)
        lib().onnd_import(self._h, ids.ctypes.data, dist.ctypes.data, fresh.ctypes.data)

    def counters(self):
        c = (ctypes.c_int64 * 3)()
        lib().onnd_counters(self._h, c)
        return {"pairs": c[0], "offered": c[1], "updates": c[2]}

    def graph(self):
        ids = np.empty((self.n, self.k), dtype=np.int32)
        dist = np.empty((self.n, self.k), dtype=np.float64)
        fresh = np.empty((self.n, self.k), dtype=np.uint8)
        lib().onnd_export(self._h, ids.ctypes.data, dist.ctypes.data, fresh.ctypes.data)
        return ids, dist, fresh
