"""Thin ctypes binding of libdynakv.so: same names as the C ABI, argument marshalling only.

torch owns device memory and streams; every step of the path runs in the library's kernels.  There is
no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdynakv.so")

DTYPES = {"f32": 0, "f16": 1, "bf16": 2}
TORCH_DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
ERR_TOKENS, ERR_CLUSTERS, ERR_SPLIT_SIZE, ERR_SELECT, ERR_INIT, ERR_IMPORT, ERR_PLACE = 1, 2, 4, 8, 16, 32, 64
OK, EINVAL, ECAPACITY, ESTATE, EHIP, ENOMEM = range(6)
SEARCH_STORAGE, SEARCH_MEAN = 0, 1
UPDATE_ADAPTIVE, UPDATE_STATIC, UPDATE_TOKENS, UPDATE_LOCAL = 0, 1, 2, 3
LAUNCH_SEPARATE, LAUNCH_SPLIT_KERNEL = 1 << 16, 1 << 17


def launch_shape(kv_splits: int = 0, att_waves: int = 0, flags: int = 0) -> int:
    """The value of Config.launch (DYNAKV_LAUNCH in the header)."""
    return (kv_splits & 255) | ((att_waves & 255) << 8) | flags


class _Cfg(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("n_units", "group_size", "head_dim", "dtype", "n_clusters_init",
                                          "max_clusters", "max_tokens", "kmeans_iters", "buffer_max",
                                          "group_reduce")] + \
               [(k, C.c_float) for k in ("var_alpha", "size_factor", "softmax_scale")] + \
               [(k, C.c_int32) for k in ("search_copy", "score_round", "update_mode", "launch", "local_window", "local_clusters")]


_STATE_FIELDS = ("n_clusters", "n_tokens", "error", "tau", "centroids", "size", "buffered", "flag", "m2", "offsets",
                 "members", "scores", "n_selected", "selected", "n_gathered", "gathered", "last_assign", "counters",
                 "keys", "values", "first_page")
# what dynakv_import_state reads
IMPORT_FIELDS = ("n_clusters", "n_tokens", "tau", "centroids", "size", "buffered", "flag", "m2", "offsets", "members",
                 "keys", "values", "n_selected", "selected")


class _State(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in _STATE_FIELDS]


@dataclass
class Config:
    n_units: int
    group_size: int
    dtype: str
    n_clusters_init: int
    max_clusters: int
    max_tokens: int
    kmeans_iters: int = 10
    buffer_max: int = 16
    group_reduce: int = 0
    var_alpha: float = 0.0
    size_factor: float = 0.0
    softmax_scale: float = 0.0
    head_dim: int = 128
    search_copy: int = SEARCH_STORAGE
    score_round: int = 0
    update_mode: int = UPDATE_ADAPTIVE
    launch: int = 0
    local_window: int = 0
    local_clusters: int = 0


_lib = None


def load():
    """Loads the built library; raises if it is missing (build it with paper_2511_07427_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libdynakv.so is not built: run `python paper_2511_07427_amd/build.py`")
        lib = C.CDLL(LIB_PATH)
        vp, i32 = C.c_void_p, C.c_int32
        lib.dynakv_workspace_bytes.restype = C.c_size_t
        lib.dynakv_workspace_bytes.argtypes = [C.POINTER(_Cfg)]
        lib.dynakv_create.argtypes = [C.POINTER(_Cfg), vp, C.c_size_t, C.POINTER(vp)]
        lib.dynakv_destroy.argtypes = [vp]
        lib.dynakv_build_index.argtypes = [vp, vp, vp, i32, vp, vp]
        lib.dynakv_extend_index.argtypes = [vp, vp, vp, i32, vp]
        lib.dynakv_place_by_coretrieval.argtypes = [vp, vp, vp, i32, vp, i32, i32, vp, vp, vp]
        lib.dynakv_retrieve_attend.argtypes = [vp, vp, i32, vp, vp, vp]
        lib.dynakv_retrieve_attend_static.argtypes = [vp, vp, i32, vp, vp, vp]
        lib.dynakv_append.argtypes = [vp, vp, vp, vp]
        lib.dynakv_split.argtypes = [vp, vp]
        lib.dynakv_decode_step.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp]
        lib.dynakv_export_state.argtypes = [vp, C.POINTER(_State), vp]
        lib.dynakv_import_state.argtypes = [vp, C.POINTER(_State), vp]
        lib.dynakv_profile_enable.argtypes = [vp, i32]
        lib.dynakv_profile_sample.argtypes = [vp, i32, i32]
        lib.dynakv_profile_read.argtypes = [vp, C.POINTER(i32), C.POINTER(C.c_double)]
        lib.dynakv_profiled_kernel.restype = C.c_char_p
        lib.dynakv_profiled_kernel.argtypes = [vp]
        lib.dynakv_strerror.restype = C.c_char_p
        lib.dynakv_strerror.argtypes = [C.c_int]
        _lib = lib
    return _lib


def _check(rc, what):
    if rc != 0:
        raise RuntimeError("%s: %s" % (what, load().dynakv_strerror(rc).decode()))


def _cfg(cfg: Config) -> _Cfg:
    return _Cfg(cfg.n_units, cfg.group_size, cfg.head_dim, DTYPES[cfg.dtype], cfg.n_clusters_init, cfg.max_clusters,
                cfg.max_tokens, cfg.kmeans_iters, cfg.buffer_max, cfg.group_reduce, cfg.var_alpha, cfg.size_factor,
                cfg.softmax_scale, cfg.search_copy, cfg.score_round, cfg.update_mode, cfg.launch, cfg.local_window,
                cfg.local_clusters)


def dynakv_workspace_bytes(cfg: Config) -> int:
    return load().dynakv_workspace_bytes(C.byref(_cfg(cfg)))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, shape=None) -> int:
    assert t.is_cuda and t.is_contiguous() and t.dtype == dtype, (t.device, t.dtype, dtype)
    if shape is not None:
        assert tuple(t.shape) == tuple(shape), (tuple(t.shape), tuple(shape))
    return t.data_ptr()


class Index:
    """One index (dynakv_index_t) over a workspace tensor it keeps alive.  Work goes to torch's current stream."""

    def __init__(self, cfg: Config, device="cuda:0"):
        self.cfg = cfg
        self._lib = load()
        self._c = _cfg(cfg)
        nbytes = self._lib.dynakv_workspace_bytes(C.byref(self._c))
        if nbytes == 0:
            raise ValueError("dynakv: invalid configuration %r" % (cfg,))
        self.device = torch.device(device)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        h = C.c_void_p()
        _check(self._lib.dynakv_create(C.byref(self._c), self.workspace.data_ptr(), nbytes, C.byref(h)), "dynakv_create")
        self._h = h
        self._tdtype = TORCH_DTYPES[cfg.dtype]

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib.dynakv_destroy(self._h)
            self._h = None

    # ---- the four calls ---------------------------------------------------------------------
    def dynakv_build_index(self, K: torch.Tensor, V: torch.Tensor, init_idx: torch.Tensor):
        c = self.cfg
        n = K.shape[1]
        kp = _dev(K, self._tdtype, (c.n_units, n, c.head_dim))
        vp = _dev(V, self._tdtype, (c.n_units, n, c.head_dim))
        ip = _dev(init_idx, torch.int32, (c.n_units, c.n_clusters_init))
        _check(self._lib.dynakv_build_index(self._h, kp, vp, n, ip, _stream()), "dynakv_build_index")

    def dynakv_extend_index(self, K: torch.Tensor, V: torch.Tensor):
        c = self.cfg
        n = K.shape[1]
        kp = _dev(K, self._tdtype, (c.n_units, n, c.head_dim))
        vp = _dev(V, self._tdtype, (c.n_units, n, c.head_dim))
        _check(self._lib.dynakv_extend_index(self._h, kp, vp, n, _stream()), "dynakv_extend_index")

    def dynakv_retrieve_attend(self, Q: torch.Tensor, token_budget: int, out: torch.Tensor, lse: torch.Tensor | None):
        c = self.cfg
        qp = _dev(Q, self._tdtype, (c.n_units, c.group_size, c.head_dim))
        op = _dev(out, torch.float32, (c.n_units, c.group_size, c.head_dim))
        lp = _dev(lse, torch.float32, (c.n_units, c.group_size)) if lse is not None else None
        _check(self._lib.dynakv_retrieve_attend(self._h, qp, int(token_budget), op, lp, _stream()),
               "dynakv_retrieve_attend")

    def dynakv_place_by_coretrieval(self, K: torch.Tensor, V: torch.Tensor, Qref: torch.Tensor, token_budget: int):
        """Returns (P [U, M0, M0] float32: Eq. 8's co-retrieval probabilities, order [U, M0] int32: the placement chain),
        both device tensors; the index's pages are laid out afresh in chain order."""
        c = self.cfg
        n, r = K.shape[1], Qref.shape[0]
        kp = _dev(K, self._tdtype, (c.n_units, n, c.head_dim))
        vp = _dev(V, self._tdtype, (c.n_units, n, c.head_dim))
        qp = _dev(Qref, self._tdtype, (r, c.n_units, c.group_size, c.head_dim))
        P = torch.empty(c.n_units, c.n_clusters_init, c.n_clusters_init, dtype=torch.float32, device=self.device)
        order = torch.empty(c.n_units, c.n_clusters_init, dtype=torch.int32, device=self.device)
        _check(self._lib.dynakv_place_by_coretrieval(self._h, kp, vp, n, qp, r, int(token_budget), P.data_ptr(),
                                                      order.data_ptr(), _stream()), "dynakv_place_by_coretrieval")
        return P, order

    def dynakv_retrieve_attend_static(self, Q: torch.Tensor, token_budget: int, out: torch.Tensor, lse: torch.Tensor | None):
        """The same retrieval with the split-KV scratch in the library's static device array; returns the status
        (ECAPACITY if the configuration needs more scratch than the array holds) instead of raising on it."""
        c = self.cfg
        qp = _dev(Q, self._tdtype, (c.n_units, c.group_size, c.head_dim))
        op = _dev(out, torch.float32, (c.n_units, c.group_size, c.head_dim))
        lp = _dev(lse, torch.float32, (c.n_units, c.group_size)) if lse is not None else None
        rc = self._lib.dynakv_retrieve_attend_static(self._h, qp, int(token_budget), op, lp, _stream())
        if rc not in (OK, ECAPACITY):
            _check(rc, "dynakv_retrieve_attend_static")
        return rc

    def dynakv_append(self, k_new: torch.Tensor, v_new: torch.Tensor):
        c = self.cfg
        kp = _dev(k_new, self._tdtype, (c.n_units, c.head_dim))
        vp = _dev(v_new, self._tdtype, (c.n_units, c.head_dim))
        _check(self._lib.dynakv_append(self._h, kp, vp, _stream()), "dynakv_append")

    def dynakv_split(self):
        _check(self._lib.dynakv_split(self._h, _stream()), "dynakv_split")

    def dynakv_decode_step(self, Q: torch.Tensor, token_budget: int, out: torch.Tensor, lse: torch.Tensor | None,
                           k_new: torch.Tensor, v_new: torch.Tensor):
        c = self.cfg
        qp = _dev(Q, self._tdtype, (c.n_units, c.group_size, c.head_dim))
        op = _dev(out, torch.float32, (c.n_units, c.group_size, c.head_dim))
        lp = _dev(lse, torch.float32, (c.n_units, c.group_size)) if lse is not None else None
        kp = _dev(k_new, self._tdtype, (c.n_units, c.head_dim))
        vp = _dev(v_new, self._tdtype, (c.n_units, c.head_dim))
        _check(self._lib.dynakv_decode_step(self._h, qp, int(token_budget), op, lp, kp, vp, _stream()),
               "dynakv_decode_step")

    def decode_step_ptrs(self, q_ptr: int, budget: int, out_ptr: int, lse_ptr: int, k_ptr: int, v_ptr: int, stream: int):
        """dynakv_decode_step on raw device addresses, without per-call tensor checks, for loops where
        interpreter time would otherwise dominate."""
        rc = self._lib.dynakv_decode_step(self._h, q_ptr, budget, out_ptr, lse_ptr, k_ptr, v_ptr, stream)
        if rc:
            _check(rc, "decode step")

    # ---- timing aid ---------------------------------------------------------------------------
    def dynakv_profile_enable(self, max_launches: int):
        _check(self._lib.dynakv_profile_enable(self._h, int(max_launches)), "dynakv_profile_enable")

    def dynakv_profile_sample(self, every: int, run: int = 1):
        _check(self._lib.dynakv_profile_sample(self._h, int(every), int(run)), "dynakv_profile_sample")

    def dynakv_profile_read(self):
        n, ms = C.c_int32(), C.c_double()
        _check(self._lib.dynakv_profile_read(self._h, C.byref(n), C.byref(ms)), "dynakv_profile_read")
        return n.value, ms.value

    def dynakv_profiled_kernel(self) -> str:
        return self._lib.dynakv_profiled_kernel(self._h).decode()

    # ---- snapshot -------------------------------------------------------------------------------
    def _state_spec(self):
        c = self.cfg
        U, M, N, d = c.n_units, c.max_clusters, c.max_tokens, c.head_dim
        i32, f32, f64, i64 = torch.int32, torch.float32, torch.float64, torch.int64
        return dict(n_clusters=((U,), i32), n_tokens=((U,), i32), error=((U,), i32), tau=((U,), f64),
                    centroids=((U, M, d), f32), size=((U, M), i32), buffered=((U, M), i32), flag=((U, M), i32),
                    m2=((U, M), f64), offsets=((U, M + 1), i32), members=((U, N), i32), scores=((U, M), f32),
                    n_selected=((U,), i32), selected=((U, M), i32), n_gathered=((U,), i32), gathered=((U, N), i32),
                    last_assign=((U,), i32), counters=((U, 8), i64), keys=((U, N, d), self._tdtype),
                    values=((U, N, d), self._tdtype), first_page=((U, M), i32))

    def dynakv_export_state(self, fields=_STATE_FIELDS[:-3], to_cpu=True):
        """Returns the requested parts of the state (the call waits for the stream), as CPU tensors unless
        to_cpu is False.  A set error word does not raise: the returned status is kept in `self.export_status`
        (ECAPACITY in that case) and the words are in the "error" field."""
        spec = self._state_spec()
        bufs = {k: torch.zeros(spec[k][0], dtype=spec[k][1], device=self.device) for k in fields}
        st = _State(**{k: (bufs[k].data_ptr() if k in bufs else None) for k in _STATE_FIELDS})
        rc = self._lib.dynakv_export_state(self._h, C.byref(st), _stream())
        self.export_status = rc
        if rc not in (OK, ECAPACITY):
            _check(rc, "dynakv_export_state")
        return {k: v.cpu() for k, v in bufs.items()} if to_cpu else bufs

    def dynakv_import_state(self, state: dict):
        """state: device tensors by field name (the fields of IMPORT_FIELDS; n_selected / selected optional), shaped
        like those dynakv_export_state returns."""
        spec = self._state_spec()
        ptrs = {}
        for k in IMPORT_FIELDS:
            if k in state:
                ptrs[k] = _dev(state[k], spec[k][1], spec[k][0])
        st = _State(**{k: ptrs.get(k) for k in _STATE_FIELDS})
        _check(self._lib.dynakv_import_state(self._h, C.byref(st), _stream()), "dynakv_import_state")
