"""Python binding of the C boundary (include/tagore_knn.h): argument marshalling only.

torch supplies device memory and the stream; every step of the method runs in the HIP
library.  There is no fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtagore_knn.so")

TG_MAX_ROUNDS = 64
METRICS = {"l2": 0, "ip": 1, "cosine": 2}


class Params(ctypes.Structure):
    _fields_ = [("k", ctypes.c_int32), ("metric", ctypes.c_int32), ("it1", ctypes.c_int32), ("it2", ctypes.c_int32),
                ("S", ctypes.c_int32), ("R", ctypes.c_int32), ("C", ctypes.c_int32), ("parts", ctypes.c_int32),
                ("m", ctypes.c_int32), ("delta", ctypes.c_float),
                ("finalize", ctypes.c_int32), ("screen", ctypes.c_int32), ("join_f16", ctypes.c_int32),
                ("seed", ctypes.c_uint64)]


class Stats(ctypes.Structure):
    _fields_ = [("rounds_phase1", ctypes.c_int32), ("rounds_phase2", ctypes.c_int32),
                ("updates", ctypes.c_int64 * TG_MAX_ROUNDS),
                ("ms_norms", ctypes.c_float), ("ms_init", ctypes.c_float), ("ms_finalize", ctypes.c_float),
                ("ms_sample", ctypes.c_float * TG_MAX_ROUNDS), ("ms_join", ctypes.c_float * TG_MAX_ROUNDS),
                ("ms_adjacency", ctypes.c_float * TG_MAX_ROUNDS),
                ("ms_update", ctypes.c_float * TG_MAX_ROUNDS),
                ("join_pairs", ctypes.c_double * TG_MAX_ROUNDS), ("join_vectors", ctypes.c_double * TG_MAX_ROUNDS),
                ("undefined_rows", ctypes.c_int64)]

    def as_dict(self):
        r = self.rounds_phase1 + self.rounds_phase2
        return dict(rounds_phase1=self.rounds_phase1, rounds_phase2=self.rounds_phase2,
                    updates=list(self.updates[:r]), ms_norms=self.ms_norms, ms_init=self.ms_init,
                    ms_finalize=self.ms_finalize, ms_sample=list(self.ms_sample[:r]), ms_join=list(self.ms_join[:r]),
                    ms_adjacency=list(self.ms_adjacency[:r]), ms_update=list(self.ms_update[:r]), join_pairs=list(self.join_pairs[:r]),
                    join_vectors=list(self.join_vectors[:r]), undefined_rows=self.undefined_rows)


EXPORTS = ["tg_knn_default_params", "tg_knn_workspace_bytes", "tg_knn_build", "tg_knn_build_ex", "tg_knn_create",
           "tg_knn_destroy", "tg_knn_init", "tg_knn_phase1_round", "tg_knn_begin_phase2", "tg_knn_phase2_round",
           "tg_knn_finalize", "tg_knn_get_stats", "tg_knn_export", "tg_knn_import", "tg_knn_sample_blocks",
           "tg_knn_join_distances", "tg_knn_block_adjacency", "tg_exact_knn", "tg_exact_knn_static", "tg_exact_knn_static_scratch_bytes", "tg_prune_rank", "tg_prune_dist", "tg_prune_angle", "tg_prune_dispersion", "tg_angle_at", "tg_merge_local", "tg_lists_clear",
           "tg_last_error"]

_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libtagore_knn.so is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32, u64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_size_t
        PP, SP = ctypes.POINTER(Params), ctypes.POINTER(Stats)
        L.tg_knn_default_params.argtypes = [i32, i32, PP]
        L.tg_knn_workspace_bytes.restype = sz
        L.tg_knn_workspace_bytes.argtypes = [i64, i32, PP]
        L.tg_knn_build.argtypes = [vp, i64, i32, i32, i32, i32, u64, vp, vp, vp]
        L.tg_knn_build_ex.argtypes = [vp, i64, i32, PP, vp, sz, vp, vp, SP, vp]
        L.tg_knn_create.argtypes = [ctypes.POINTER(vp), vp, i64, i32, PP, vp, sz, vp]
        L.tg_knn_destroy.argtypes = [vp]
        L.tg_knn_init.argtypes = [vp]
        L.tg_knn_phase1_round.argtypes = [vp, ctypes.POINTER(i64)]
        L.tg_knn_begin_phase2.argtypes = [vp]
        L.tg_knn_phase2_round.argtypes = [vp, ctypes.POINTER(i64)]
        L.tg_knn_finalize.argtypes = [vp, vp, vp]
        L.tg_knn_get_stats.argtypes = [vp, SP]
        L.tg_knn_export.argtypes = [vp, vp, vp, vp]
        L.tg_knn_import.argtypes = [vp, vp, vp, vp]
        L.tg_knn_sample_blocks.argtypes = [vp, vp, vp]
        L.tg_knn_join_distances.argtypes = [vp, vp, vp, i64, vp]
        L.tg_knn_block_adjacency.argtypes = [vp, vp]
        L.tg_exact_knn.argtypes = [vp, i64, i32, i32, i32, vp, i64, vp, vp, vp]
        L.tg_exact_knn_static.argtypes = [vp, i64, i32, i32, i32, vp, i64, vp, vp, vp]
        L.tg_exact_knn_static_scratch_bytes.restype = sz
        L.tg_exact_knn_static_scratch_bytes.argtypes = []
        L.tg_prune_rank.argtypes = [vp, i64, i32, i32, vp, vp, vp]
        L.tg_merge_local.argtypes = [vp, vp, i64, i32, vp, vp, i64, i32, vp, vp]
        L.tg_lists_clear.argtypes = [vp, vp, i64, i32, vp]
        L.tg_prune_dist.argtypes = [vp, i64, i32, vp, i32, i32, i32, ctypes.c_float, i32, vp, vp, vp]
        L.tg_prune_angle.argtypes = [vp, i64, i32, vp, i32, i32, i32, ctypes.c_float, i32, vp, vp, vp]
        L.tg_prune_dispersion.argtypes = [vp, i64, i32, vp, i32, i32, i32, i32, vp, vp, vp]
        L.tg_angle_at.argtypes = [vp, vp, vp, vp, i64, vp]
        L.tg_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


class TagoreError(RuntimeError):
    pass


def _check(rc):
    if rc != 0:
        raise TagoreError("tagore_knn error %d: %s" % (rc, lib().tg_last_error().decode()))


def _stream_ptr():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_f32(X):
    if not (isinstance(X, torch.Tensor) and X.is_cuda and X.dtype == torch.float32 and X.dim() == 2 and X.is_contiguous()):
        raise TypeError("X must be a contiguous 2-D float32 CUDA tensor")
    return X


def default_params(k, iters=0, metric="l2", seed=1, **overrides) -> Params:
    p = Params()
    _check(lib().tg_knn_default_params(k, iters, ctypes.byref(p)))
    p.metric = METRICS[metric] if isinstance(metric, str) else int(metric)
    p.seed = seed
    for name, val in overrides.items():
        if not hasattr(p, name):
            raise AttributeError(name)
        setattr(p, name, val)
    return p


def workspace_bytes(n, d, params: Params) -> int:
    b = lib().tg_knn_workspace_bytes(n, d, ctypes.byref(params))
    if b == 0:
        raise TagoreError("invalid problem: %s" % lib().tg_last_error().decode())
    return b


def knn_build(X, k, metric="l2", iters=0, seed=1):
    """tg_knn_build: the whole of Algorithm 1; returns (ids int32 n x k, dist fp32 n x k)."""
    X = _dev_f32(X)
    n, d = X.shape
    ids = torch.empty((n, k), dtype=torch.int32, device=X.device)
    dist = torch.empty((n, k), dtype=torch.float32, device=X.device)
    _check(lib().tg_knn_build(X.data_ptr(), n, d, k, METRICS[metric], iters, seed, ids.data_ptr(), dist.data_ptr(),
                              _stream_ptr()))
    return ids, dist


def knn_build_ex(X, params: Params, workspace=None, want_stats=True):
    """tg_knn_build_ex with a torch-owned workspace; returns (ids, dist, stats dict or None)."""
    X = _dev_f32(X)
    n, d = X.shape
    if workspace is None:
        workspace = torch.empty(workspace_bytes(n, d, params), dtype=torch.uint8, device=X.device)
    ids = torch.empty((n, params.k), dtype=torch.int32, device=X.device)
    dist = torch.empty((n, params.k), dtype=torch.float32, device=X.device)
    st = Stats() if want_stats else None
    _check(lib().tg_knn_build_ex(X.data_ptr(), n, d, ctypes.byref(params), workspace.data_ptr(), workspace.numel(),
                                 ids.data_ptr(), dist.data_ptr(), ctypes.byref(st) if st is not None else None,
                                 _stream_ptr()))
    return ids, dist, (st.as_dict() if st is not None else None)


class Builder:
    """The step-by-step calls of the boundary (tg_knn_create ... tg_knn_destroy)."""

    def __init__(self, X, params: Params):
        self.X = _dev_f32(X)
        self.n, self.d = self.X.shape
        self.params = params
        self.k = params.k
        self.workspace = torch.empty(workspace_bytes(self.n, self.d, params), dtype=torch.uint8, device=X.device)
        h = ctypes.c_void_p()
        _check(lib().tg_knn_create(ctypes.byref(h), self.X.data_ptr(), self.n, self.d, ctypes.byref(params),
                                   self.workspace.data_ptr(), self.workspace.numel(), _stream_ptr()))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            torch.cuda.synchronize()
            lib().tg_knn_destroy(self._h)
            self._h = None

    __del__ = close

    def init(self):
        _check(lib().tg_knn_init(self._h))

    def phase1_round(self, want_updates=True):
        u = ctypes.c_int64(-1)
        _check(lib().tg_knn_phase1_round(self._h, ctypes.byref(u) if want_updates else None))
        return u.value

    def begin_phase2(self):
        _check(lib().tg_knn_begin_phase2(self._h))

    def phase2_round(self, want_updates=True):
        u = ctypes.c_int64(-1)
        _check(lib().tg_knn_phase2_round(self._h, ctypes.byref(u) if want_updates else None))
        return u.value

    def finalize(self):
        ids = torch.empty((self.n, self.k), dtype=torch.int32, device=self.X.device)
        dist = torch.empty((self.n, self.k), dtype=torch.float32, device=self.X.device)
        _check(lib().tg_knn_finalize(self._h, ids.data_ptr(), dist.data_ptr()))
        return ids, dist

    def stats(self):
        st = Stats()
        _check(lib().tg_knn_get_stats(self._h, ctypes.byref(st)))
        return st.as_dict()

    def graph(self):
        """Current lists: (ids int32, dist fp32, fresh uint8), each n x k."""
        dev = self.X.device
        ids = torch.empty((self.n, self.k), dtype=torch.int32, device=dev)
        dist = torch.empty((self.n, self.k), dtype=torch.float32, device=dev)
        fresh = torch.empty((self.n, self.k), dtype=torch.uint8, device=dev)
        _check(lib().tg_knn_export(self._h, ids.data_ptr(), dist.data_ptr(), fresh.data_ptr()))
        return ids, dist, fresh

    def set_graph(self, ids, dist, fresh):
        dev = self.X.device
        ids = ids.to(device=dev, dtype=torch.int32).contiguous()
        dist = dist.to(device=dev, dtype=torch.float32).contiguous()
        fresh = fresh.to(device=dev, dtype=torch.uint8).contiguous()
        assert ids.shape == dist.shape == fresh.shape == (self.n, self.k)
        if int(ids.min()) < 0 or int(ids.max()) >= self.n:
            raise ValueError("ids out of range")
        _check(lib().tg_knn_import(self._h, ids.data_ptr(), dist.data_ptr(), fresh.data_ptr()))
        torch.cuda.current_stream().synchronize()

    def sample_blocks(self):
        """Blocks of the coming phase-1 round: (blk int32 n x 128, sizes int32 n x 2)."""
        dev = self.X.device
        blk = torch.empty((self.n, 128), dtype=torch.int32, device=dev)
        sizes = torch.empty((self.n, 2), dtype=torch.int32, device=dev)
        _check(lib().tg_knn_sample_blocks(self._h, blk.data_ptr(), sizes.data_ptr()))
        return blk, sizes

    def block_adjacency(self):
        """For the blocks last sampled: uint32 n x 128 x 4, bit x of entry (v, p) = position x of v's block is in position p's list."""
        adj = torch.zeros((self.n, 128, 4), dtype=torch.int32, device=self.X.device)
        _check(lib().tg_knn_block_adjacency(self._h, adj.data_ptr()))
        return adj

    def join_distances(self, blk, sizes):
        dev = self.X.device
        blk = blk.to(device=dev, dtype=torch.int32).contiguous()
        sizes = sizes.to(device=dev, dtype=torch.int32).contiguous()
        nb = blk.shape[0]
        assert blk.shape == (nb, 128) and sizes.shape == (nb, 2)
        out = torch.full((nb, 64, 128), float("nan"), dtype=torch.float32, device=dev)
        _check(lib().tg_knn_join_distances(self._h, blk.data_ptr(), sizes.data_ptr(), nb, out.data_ptr()))
        return out


def prune_rank(ids, d_out, want_counts=False):
    """tg_prune_rank: the d_out neighbours of every row with the fewest detourable routes."""
    if not (ids.is_cuda and ids.dtype == torch.int32 and ids.dim() == 2 and ids.is_contiguous()):
        raise ValueError("ids must be a contiguous int32 CUDA tensor of shape (n, k)")
    n, k = ids.shape
    out = torch.empty((n, d_out), dtype=torch.int32, device=ids.device)
    cnt = torch.empty((n, k), dtype=torch.int32, device=ids.device) if want_counts else None
    _check(lib().tg_prune_rank(ids.data_ptr(), n, k, d_out, out.data_ptr(), cnt.data_ptr() if want_counts else None,
                               _stream_ptr()))
    return (out, cnt) if want_counts else out


def prune_angle(X, ids, d_out, gamma_deg=60.0, hops=1, cand_size=64, want_degrees=False):
    """tg_prune_angle: NSSG pruning (angles above gamma_deg between kept neighbours) over the 1-hop or 2-hop candidates."""
    return _prune_filter("tg_prune_angle", X, ids, d_out, gamma_deg, hops, cand_size, want_degrees)


def prune_dist(X, ids, d_out, alpha=1.0, hops=1, cand_size=64, want_degrees=False):
    """tg_prune_dist: NSG (alpha = 1) / Vamana (alpha > 1) pruning over the 1-hop or 2-hop candidates."""
    return _prune_filter("tg_prune_dist", X, ids, d_out, alpha, hops, cand_size, want_degrees)


def prune_dispersion(X, ids, d_out, hops=1, cand_size=64, want_degrees=False):
    """tg_prune_dispersion: DPG pruning (greedy choice of the neighbours whose angles at the node add up to the most)."""
    return _prune_filter("tg_prune_dispersion", X, ids, d_out, None, hops, cand_size, want_degrees)


def angle_at(a, b, c):
    """tg_angle_at: the angle (radians) between two directions from squared lengths, elementwise."""
    for v in (a, b, c):
        if not (isinstance(v, torch.Tensor) and v.is_cuda and v.dtype == torch.float32 and v.dim() == 1 and v.is_contiguous()):
            raise TypeError("a, b, c must be contiguous 1-D float32 CUDA tensors")
    if not (a.numel() == b.numel() == c.numel()):
        raise ValueError("a, b, c must have the same number of elements")
    out = torch.empty_like(a)
    _check(lib().tg_angle_at(a.data_ptr(), b.data_ptr(), c.data_ptr(), out.data_ptr(), a.numel(), _stream_ptr()))
    return out


def _prune_filter(entry, X, ids, d_out, thres, hops, cand_size, want_degrees):
    X = _dev_f32(X)
    if not (ids.is_cuda and ids.dtype == torch.int32 and ids.dim() == 2 and ids.is_contiguous()):
        raise ValueError("ids must be a contiguous int32 CUDA tensor of shape (n, k)")
    n, k = ids.shape
    if X.shape[0] != n:
        raise ValueError("X and ids disagree on n")
    out = torch.empty((n, d_out), dtype=torch.int32, device=ids.device)
    deg = torch.empty(n, dtype=torch.int32, device=ids.device) if want_degrees else None
    rule = () if thres is None else (float(thres),)
    _check(getattr(lib(), entry)(X.data_ptr(), n, X.shape[1], ids.data_ptr(), k, hops, cand_size, *rule, d_out,
                                 out.data_ptr(), deg.data_ptr() if want_degrees else None, _stream_ptr()))
    return (out, deg) if want_degrees else out


def lists_clear(n, k, device="cuda"):
    """New n x k lists with every entry unused (tg_lists_clear): ids -1, distances +inf."""
    ids = torch.empty((n, k), dtype=torch.int32, device=device)
    dist = torch.empty((n, k), dtype=torch.float32, device=device)
    _check(lib().tg_lists_clear(ids.data_ptr(), dist.data_ptr(), n, k, _stream_ptr()))
    return ids, dist


def merge_local(g_ids, g_dist, l_ids, l_dist, local_to_global):
    """tg_merge_local: merges a local index (local numbering) into the global lists, in place."""
    for t_, dt in ((g_ids, torch.int32), (g_dist, torch.float32), (l_ids, torch.int32), (l_dist, torch.float32),
                   (local_to_global, torch.int32)):
        if not (t_.is_cuda and t_.dtype == dt and t_.is_contiguous()):
            raise ValueError("arguments must be contiguous CUDA tensors (ids int32, distances float32)")
    n, k = g_ids.shape
    nl, kl = l_ids.shape
    if g_dist.shape != g_ids.shape or l_dist.shape != l_ids.shape or local_to_global.numel() != nl:
        raise ValueError("shapes disagree")
    _check(lib().tg_merge_local(g_ids.data_ptr(), g_dist.data_ptr(), n, k, l_ids.data_ptr(), l_dist.data_ptr(), nl, kl,
                                local_to_global.data_ptr(), _stream_ptr()))


def exact_knn_static(X, k, metric="l2", rows=None, out=None):
    """tg_exact_knn_static: tg_exact_knn on the library's static scratch (the call itself allocates nothing;
    pass ``out = (ids, dist)`` to keep torch from allocating the outputs here)."""
    X = _dev_f32(X)
    n, d = X.shape
    if rows is None:
        nq, rp = n, None
    else:
        if not (rows.is_cuda and rows.dtype == torch.int64 and rows.is_contiguous()):
            raise TypeError("rows must be a contiguous int64 CUDA tensor")
        nq, rp = rows.numel(), rows.data_ptr()
    if out is None:
        out = (torch.empty((nq, k), dtype=torch.int32, device=X.device), torch.empty((nq, k), dtype=torch.float32, device=X.device))
    ids, dist = out
    if not (ids.is_cuda and ids.dtype == torch.int32 and ids.is_contiguous() and tuple(ids.shape) == (nq, k)
            and dist.is_cuda and dist.dtype == torch.float32 and dist.is_contiguous() and tuple(dist.shape) == (nq, k)):
        raise TypeError("out must be (int32, float32) contiguous CUDA tensors of shape (nq, k)")
    _check(lib().tg_exact_knn_static(X.data_ptr(), n, d, k, METRICS[metric], rp, nq, ids.data_ptr(), dist.data_ptr(),
                                     _stream_ptr()))
    return ids, dist


def exact_knn(X, k, metric="l2", rows=None):
    """tg_exact_knn: exhaustive k-NN of the given rows (all rows if None)."""
    X = _dev_f32(X)
    n, d = X.shape
    if rows is None:
        nq, rp, keep = n, None, None
    else:
        keep = rows.to(device=X.device, dtype=torch.int64).contiguous()
        nq, rp = keep.numel(), keep.data_ptr()
    ids = torch.empty((nq, k), dtype=torch.int32, device=X.device)
    dist = torch.empty((nq, k), dtype=torch.float32, device=X.device)
    _check(lib().tg_exact_knn(X.data_ptr(), n, d, k, METRICS[metric], rp, nq, ids.data_ptr(), dist.data_ptr(),
                              _stream_ptr()))
    return ids, dist
