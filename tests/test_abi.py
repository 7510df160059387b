"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared symbol, sizes
workspaces, and rejects misuse with status codes before anything is enqueued."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2511_07427_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_07427_amd.build import build
        build()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "dynakv.h")).read()
    names = set(re.findall(r"\b(dynakv_[a-z_]+)\s*\(", hdr))
    assert {"dynakv_build_index", "dynakv_append", "dynakv_split", "dynakv_retrieve_attend"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), n


def test_struct_sizes_match_the_header():
    assert C.sizeof(binding._Cfg) == 19 * 4
    assert C.sizeof(binding._State) == 21 * 8


def _cfg(**kw):
    base = dict(n_units=2, group_size=4, dtype="f16", n_clusters_init=8, max_clusters=32, max_tokens=256)
    base.update(kw)
    return binding.Config(**base)


def test_workspace_bytes_and_invalid_configs(lib):
    a = binding.dynakv_workspace_bytes(_cfg())
    b = binding.dynakv_workspace_bytes(_cfg(n_units=4))
    c = binding.dynakv_workspace_bytes(_cfg(dtype="f32"))
    assert 0 < a < b and a < c and a % 256 == 0
    for bad in (dict(n_units=0), dict(group_size=17), dict(head_dim=64), dict(max_clusters=4), dict(max_clusters=131073), dict(n_clusters_init=8193, max_clusters=9000, max_tokens=9000), dict(search_copy=2),
                dict(score_round=2), dict(update_mode=9), dict(update_mode=3), dict(update_mode=3, local_window=200, local_clusters=4), dict(local_window=8), dict(launch=1 << 20), dict(launch=3 << 8),
                dict(kmeans_iters=0), dict(buffer_max=-1), dict(group_reduce=2), dict(max_tokens=4),
                dict(softmax_scale=-1.0)):
        assert binding.dynakv_workspace_bytes(_cfg(**bad)) == 0, bad


def test_create_and_call_order_errors(lib):
    cfg = binding._cfg(_cfg())
    n = lib.dynakv_workspace_bytes(C.byref(cfg))
    h = C.c_void_p()
    fake = 1 << 20     # create only records the address; nothing is dereferenced without a GPU call
    assert lib.dynakv_create(C.byref(cfg), None, n, C.byref(h)) == 1
    assert lib.dynakv_create(C.byref(cfg), fake + 8, n, C.byref(h)) == 1          # misaligned
    assert lib.dynakv_create(C.byref(cfg), fake, n - 1, C.byref(h)) == 2          # too small
    assert lib.dynakv_create(C.byref(cfg), fake, n, C.byref(h)) == 0 and h.value
    assert lib.dynakv_retrieve_attend(h, fake, 16, fake, None, None) == 3          # before build_index
    assert lib.dynakv_append(h, fake, fake, None) == 3
    assert lib.dynakv_split(h, None) == 3
    assert lib.dynakv_build_index(h, fake, fake, 4, fake, None) == 1               # fewer tokens than clusters
    assert lib.dynakv_build_index(h, fake, fake, 512, fake, None) == 1             # more than max_tokens
    assert lib.dynakv_build_index(h, fake, None, 64, fake, None) == 1
    assert lib.dynakv_destroy(h) == 0
    assert lib.dynakv_strerror(3).decode().startswith("call out of order")


def test_page_and_centroid_table_layouts_are_bijections():
    """The index formulas of csrc/common.hpp, retyped here only to check that they tile their arrays exactly once:
    a page (K rows, then V rows, one row of 128 per token slot) and the two lane-interleaved centroid tables
    (float32 master [tile of 64][d/4][64][4]; 16-bit search copy in matrix-core operand order, [tile of 16][chunk of
    32 coordinates][16 * slice of 8 + cluster][8])."""
    def k(s_, d): return s_ * 128 + d
    def v(s_, d): return 2048 + s_ * 128 + d
    idx = [f(s_, d) for f in (k, v) for s_ in range(16) for d in range(128)]
    assert sorted(idx) == list(range(4096))
    def r(j, d): return ((j >> 6) * 32 + (d >> 2)) * 256 + (j & 63) * 4 + (d & 3)
    def rq(j, d): return (((j >> 4) * 4 + (d >> 5)) * 64 + ((d >> 3) & 3) * 16 + (j & 15)) * 8 + (d & 7)
    for f in (r, rq):
        idx = [f(j, d) for j in range(192) for d in range(128)]
        assert sorted(idx) == list(range(192 * 128))


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU's throughput; asked for more it says so and exits before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
