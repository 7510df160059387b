"""ctypes front end of the CPU oracle (test infrastructure, not the product).

Only tests, the smoke check and the CPU-baseline leg of the benchmark may import this.
It imports nothing from the GPU package.  Arrays are numpy; K/V/Q are float32 values that
the caller has already rounded to the storage type under test.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dynakv_oracle.cpp")
_LIB = os.path.join(_HERE, "libdynakv_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no fast-math, no contraction; fma() is explicit in the source)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        flags = ["-O2", "-std=c++17", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-Wall"]
        try:
            with open("/proc/cpuinfo") as f:
                if " fma " in f.read():
                    flags.append("-mfma")  # lets std::fma compile to one instruction; results are identical
        except OSError:
            pass
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["g++", *flags, _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("n_units", "group_size", "head_dim", "n_clusters_init", "max_clusters",
                                          "max_tokens", "kmeans_iters", "buffer_max", "group_reduce")] + \
               [(k, C.c_float) for k in ("var_alpha", "size_factor", "softmax_scale")] + \
               [(k, C.c_int32) for k in ("dtype", "search_copy", "score_round", "update_mode", "local_window", "local_clusters")]


@dataclass
class OracleConfig:
    n_units: int
    group_size: int
    head_dim: int
    n_clusters_init: int
    max_clusters: int
    max_tokens: int
    kmeans_iters: int = 10
    buffer_max: int = 16
    group_reduce: int = 0
    var_alpha: float = 0.0
    size_factor: float = 0.0
    softmax_scale: float = 0.0
    dtype: str = "f32"          # storage type of K, V, Q ("f32" | "f16" | "bf16")
    search_copy: int = 0        # 0: searches read the centroids rounded to the storage type; 1: the float32 means
    score_round: int = 0        # 1: cluster scores are rounded to float32 before they are ordered
    update_mode: int = 0        # 0: Algorithm 1; 1: static update; 2: every entry its own cluster; 3: local update
    local_window: int = 0       # update_mode 3: entries per local clustering
    local_clusters: int = 0     # update_mode 3: clusters it forms


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        lib.oracle_create.restype = C.c_void_p
        lib.oracle_create.argtypes = [C.POINTER(_Cfg)]
        lib.oracle_destroy.argtypes = [C.c_void_p]
        lib.oracle_set_threads.argtypes = [C.c_void_p, C.c_int]
        lib.oracle_threads_used.argtypes = [C.c_void_p]
        lib.oracle_build_index.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        lib.oracle_retrieve_attend.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        lib.oracle_append.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        lib.oracle_split.argtypes = [C.c_void_p]
        lib.oracle_extend.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        lib.oracle_coretrieval.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        for f in ("oracle_num_clusters", "oracle_num_tokens", "oracle_error", "oracle_last_assign"):
            getattr(lib, f).argtypes = [C.c_void_p, C.c_int]
        lib.oracle_tau.argtypes = [C.c_void_p, C.c_int]
        lib.oracle_tau.restype = C.c_double
        lib.oracle_get_clusters.argtypes = [C.c_void_p, C.c_int] + [C.c_void_p] * 5
        lib.oracle_get_search_copy.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        lib.oracle_round_to_storage.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int]
        lib.oracle_get_members.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        lib.oracle_get_selected.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int]
        lib.oracle_get_gather.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int]
        lib.oracle_get_scores.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        lib.oracle_get_kmeans_margins.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        lib.oracle_get_kv.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        lib.oracle_last_split_rounds.argtypes = [C.c_void_p, C.c_int]
        lib.oracle_import_unit.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int] + \
            [C.c_void_p] * 7 + [C.c_double, C.c_int, C.c_void_p]
        lib.oracle_get_diagnostics.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data


class Oracle:
    """One index over `n_units` independent units, driven call by call like the GPU library."""

    def __init__(self, cfg: OracleConfig, threads: int = 0):
        self.cfg = cfg
        self._lib = _load()
        c = _Cfg(**{k: getattr(cfg, k) for k, _ in _Cfg._fields_ if k != "dtype"},
                 dtype={"f32": 0, "f16": 1, "bf16": 2}[cfg.dtype])
        self._h = self._lib.oracle_create(C.byref(c))
        if threads:
            self._lib.oracle_set_threads(self._h, threads)

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib.oracle_destroy(self._h)
            self._h = None

    @property
    def threads_used(self) -> int:
        return self._lib.oracle_threads_used(self._h)

    # ---- the four calls -------------------------------------------------------------------
    def build_index(self, K, V, init_idx):
        """K, V: [U, N0, d]; init_idx [U, M0]: positions of the M0 distinct keys that start as centres.
        Returns the k-means objective per unit and iteration, [U, iters]."""
        K, kp = _f32(K)
        V, vp = _f32(V)
        U, N0, d = K.shape
        assert (U, d) == (self.cfg.n_units, self.cfg.head_dim) and V.shape == K.shape
        init_idx = np.ascontiguousarray(init_idx, dtype=np.int32)
        assert init_idx.shape == (U, self.cfg.n_clusters_init)
        J = np.zeros((U, self.cfg.kmeans_iters), dtype=np.float64)
        rc = self._lib.oracle_build_index(self._h, kp, vp, N0, init_idx.ctypes.data, J.ctypes.data)
        if rc:
            raise ValueError("oracle_build_index: invalid sizes or initial positions")
        return J

    def import_unit(self, u, K, V, centroids, n, b, flag, M2, offsets, members, tau, selected=()):
        """Replaces the state of unit u: K, V [N, d] by token position; per-cluster arrays of length M; members of
        cluster j = members[offsets[j]:offsets[j+1]] in storage order; `selected` = ids of the last active set."""
        K, kp = _f32(K)
        V, vp = _f32(V)
        r, rp = _f32(centroids)
        M, N = len(n), K.shape[0]
        i32 = lambda a: np.ascontiguousarray(a, dtype=np.int32)
        n, b, flag, offsets, members, selected = (i32(a) for a in (n, b, flag, offsets, members, selected))
        M2 = np.ascontiguousarray(M2, dtype=np.float64)
        assert r.shape == (M, self.cfg.head_dim) and len(offsets) == M + 1 and len(members) >= N
        rc = self._lib.oracle_import_unit(self._h, u, N, kp, vp, M, rp, n.ctypes.data, b.ctypes.data, flag.ctypes.data,
                                          M2.ctypes.data, offsets.ctypes.data, members.ctypes.data, float(tau),
                                          len(selected), selected.ctypes.data)
        if rc:
            raise ValueError("oracle_import_unit: inconsistent state")

    def retrieve_attend(self, Q, budget: int):
        """Q: [U, G, d].  Returns (out [U, G, d] float64, lse [U, G] float64)."""
        Q, qp = _f32(Q)
        U, G, d = Q.shape
        assert (U, G, d) == (self.cfg.n_units, self.cfg.group_size, self.cfg.head_dim)
        out = np.zeros((U, G, d), dtype=np.float64)
        lse = np.zeros((U, G), dtype=np.float64)
        self._lib.oracle_retrieve_attend(self._h, qp, int(budget), out.ctypes.data, lse.ctypes.data)
        return out, lse

    def append(self, k, v):
        k, kp = _f32(k)
        v, vp = _f32(v)
        assert k.shape == (self.cfg.n_units, self.cfg.head_dim) and v.shape == k.shape
        self._lib.oracle_append(self._h, kp, vp)

    def split(self):
        self._lib.oracle_split(self._h)

    def coretrieval(self, Qref, budget: int):
        """Qref: [n_ref, U, G, d] reference queries.  Returns (P [U, M, M] float64: co-retrieval probabilities of Eq. 8,
        order [U, M]: the placement chain)."""
        Q, qp = _f32(Qref)
        U, M = self.cfg.n_units, self.num_clusters(0)
        assert Q.shape[1:] == (U, self.cfg.group_size, self.cfg.head_dim)
        P = np.zeros((U, M, M), np.float64)
        order = np.zeros((U, M), np.int32)
        if self._lib.oracle_coretrieval(self._h, qp, Q.shape[0], int(budget), P.ctypes.data, order.ctypes.data):
            raise ValueError("oracle_coretrieval: units with different cluster counts")
        return P, order

    def extend(self, K, V):
        """K, V: [U, n, d]: n more prefill entries per unit, clustered adaptively one by one (every cluster resident)."""
        K, kp = _f32(K)
        V, vp = _f32(V)
        assert K.shape[0] == self.cfg.n_units and K.shape[2] == self.cfg.head_dim and V.shape == K.shape
        self._lib.oracle_extend(self._h, kp, vp, K.shape[1])

    # ---- state ------------------------------------------------------------------------------
    def num_clusters(self, u): return self._lib.oracle_num_clusters(self._h, u)
    def num_tokens(self, u): return self._lib.oracle_num_tokens(self._h, u)
    def error(self, u): return self._lib.oracle_error(self._h, u)
    def tau(self, u): return self._lib.oracle_tau(self._h, u)
    def last_assign(self, u): return self._lib.oracle_last_assign(self._h, u)

    def clusters(self, u):
        """dict(centroids [M, d] f32, n, b, flag [M] i32, M2 [M] f64)."""
        M, d = self.num_clusters(u), self.cfg.head_dim
        r = np.zeros((M, d), np.float32)
        n, b, f = (np.zeros(M, np.int32) for _ in range(3))
        M2 = np.zeros(M, np.float64)
        self._lib.oracle_get_clusters(self._h, u, r.ctypes.data, n.ctypes.data, b.ctypes.data, f.ctypes.data,
                                      M2.ctypes.data)
        return dict(centroids=r, n=n, b=b, flag=f, M2=M2)

    def search_copy(self, u):
        """[M, d] float32: every centroid rounded to the storage type, as the searches read it."""
        out = np.zeros((self.num_clusters(u), self.cfg.head_dim), dtype=np.float32)
        self._lib.oracle_get_search_copy(self._h, u, out.ctypes.data)
        return out

    def members(self, u):
        """(offsets [M+1], positions [N]): members of cluster j are positions[offsets[j]:offsets[j+1]]."""
        M, N = self.num_clusters(u), self.num_tokens(u)
        off = np.zeros(M + 1, np.int32)
        mem = np.zeros(max(N, 1), np.int32)
        self._lib.oracle_get_members(self._h, u, off.ctypes.data, mem.ctypes.data)
        return off, mem[:N]

    def labels(self, u):
        off, mem = self.members(u)
        lab = np.full(self.num_tokens(u), -1, np.int32)
        for j in range(len(off) - 1):
            lab[mem[off[j]:off[j + 1]]] = j
        return lab

    def selected(self, u):
        ids = np.zeros(max(self.num_clusters(u), 1), np.int32)
        n = self._lib.oracle_get_selected(self._h, u, ids.ctypes.data, len(ids))
        return ids[:n]

    def gather(self, u):
        pos = np.zeros(max(self.num_tokens(u), 1), np.int32)
        n = self._lib.oracle_get_gather(self._h, u, pos.ctypes.data, len(pos))
        return pos[:n]

    def scores(self, u):
        """float64 cluster scores of the last retrieval (already rounded to float32 values if score_round is set)."""
        s = np.zeros(self.num_clusters(u), np.float64)
        self._lib.oracle_get_scores(self._h, u, s.ctypes.data)
        return s

    def kv(self, u):
        """(K, V), each [N, d] float32 by token position."""
        N, d = self.num_tokens(u), self.cfg.head_dim
        K, V = np.zeros((N, d), np.float32), np.zeros((N, d), np.float32)
        self._lib.oracle_get_kv(self._h, u, K.ctypes.data, V.ctypes.data)
        return K, V

    def kmeans_margins(self, u, n0):
        m = np.zeros(n0, np.float64)
        self._lib.oracle_get_kmeans_margins(self._h, u, m.ctypes.data)
        return m

    def last_split_rounds(self, u): return self._lib.oracle_last_split_rounds(self._h, u)

    def diagnostics(self, u):
        mg = np.zeros(4, np.float64)
        ties = np.zeros(5, np.int64)
        ev = np.zeros(3, np.int64)
        self._lib.oracle_get_diagnostics(self._h, u, mg.ctypes.data, ties.ctypes.data, ev.ctypes.data)
        return dict(margin_assign=mg[0], margin_trigger=mg[1], margin_select=mg[2], margin_split=mg[3],
                    ties=dict(zip(("kmeans", "assign", "trigger", "select", "split_side"), ties.tolist())),
                    splits=int(ev[0]), failed_splits=int(ev[1]), forced_splits=int(ev[2]))


def round_to_storage(x, dtype: str):
    """The oracle's own rounding of float32 values to a storage type (nearest, ties to even), as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty_like(x)
    _load().oracle_round_to_storage(x.ctypes.data, out.ctypes.data, x.size, {"f32": 0, "f16": 1, "bf16": 2}[dtype])
    return out
