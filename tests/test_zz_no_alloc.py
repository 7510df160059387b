"""The allocation-free retrieval entry point (dynakv_retrieve_attend_static) against dynakv_retrieve_attend:
same kernels, split-KV scratch in the library's static device array instead of the caller's workspace.
Collected last so that a failure here hides no other test."""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

from parity import DEV, to_dev  # noqa: E402
from paper_2511_07427_amd import binding  # noqa: E402
from paper_2511_07427_amd.binding import LAUNCH_SEPARATE, launch_shape  # noqa: E402
from paper_2511_07427_amd.workload import CONFIGS, generate  # noqa: E402

pytestmark = pytest.mark.gpu


def _index(spec, units, steps, launch):
    w = generate(spec, units=units, steps=steps)
    U = len(units)
    ix = binding.Index(binding.Config(U, spec.group_size, spec.dtype, spec.n_clusters_init, spec.max_clusters,
                                      spec.prefill + steps, 3, 16, 0, spec.var_alpha, 0.0, 0.0, launch=launch), DEV)
    ix.dynakv_build_index(to_dev(w["K0"], spec.dtype), to_dev(w["V0"], spec.dtype), torch.from_numpy(w["init_idx"]).to(DEV))
    Kd, Vd = to_dev(w["Knew"], spec.dtype), to_dev(w["Vnew"], spec.dtype)
    for t in range(steps):
        ix.dynakv_append(Kd[t], Vd[t])
        ix.dynakv_split()
    return ix, to_dev(w["Q"], spec.dtype)


def _both(ix, Q, budget):
    c = ix.cfg
    oa = torch.empty(c.n_units, c.group_size, 128, device=DEV)
    la = torch.empty(c.n_units, c.group_size, device=DEV)
    ob, lb = torch.full_like(oa, float("nan")), torch.full_like(la, float("nan"))
    ix.dynakv_retrieve_attend(Q, budget, oa, la)
    sa = ix.dynakv_export_state(["n_selected", "selected", "n_gathered", "gathered", "scores"])
    assert ix.dynakv_retrieve_attend_static(Q, budget, ob, lb) == binding.OK
    sb = ix.dynakv_export_state(["n_selected", "selected", "n_gathered", "gathered", "scores"])
    for k in sa:                                   # integer results bit for bit
        assert torch.equal(sa[k], sb[k]), k
    oa, ob, la, lb = (x.cpu().numpy() for x in (oa, ob, la, lb))
    den = np.maximum(np.abs(oa).max(-1), 1e-6)     # values to the bar of the parity tests
    assert np.isfinite(ob).all() and (np.abs(ob - oa).max(-1) / den).max() <= 2e-3
    assert np.abs(lb - la).max() <= 2e-3
    return int(sa["n_gathered"].min())


def test_static_scratch_retrieval_matches_the_workspace_one_on_two_calls_in_a_row():
    # first a larger input (3 units, 4 workgroups per unit share the gather), then a smaller one (2 units, fewer
    # tokens, 2 workgroups per unit): the second call finds the first one's leftovers in the array
    big = CONFIGS["llama3_8b"].scaled(prefill=2048, n_clusters_init=96, budget=700)
    small = CONFIGS["qwen25_7b"].scaled(prefill=512, n_clusters_init=24, budget=150)
    ix1, Q1 = _index(big, [0, 1, 2], 24, launch_shape(4, 8, LAUNCH_SEPARATE))
    ix2, Q2 = _index(small, [0, 1], 8, launch_shape(2, 4, LAUNCH_SEPARATE))
    assert _both(ix1, Q1[5], 700) > 300
    assert _both(ix2, Q2[3], 150) > 50
    assert _both(ix1, Q1[6], 64) > 0               # and back to the first index with a small budget


def test_static_scratch_retrieval_rejects_what_does_not_fit():
    spec = CONFIGS["tiny"]
    c = binding.Config(2048, 16, "f16", 2, 4, 64, 1, 16, 0, 0.0, 0.0, 0.0, launch=launch_shape(8, 4, LAUNCH_SEPARATE))
    ix = binding.Index(c, DEV)                      # 2048 units x 8 workgroups x 16 heads x 520 B > 8 MiB
    Q = torch.zeros(2048, 16, 128, dtype=torch.float16, device=DEV)
    out = torch.zeros(2048, 16, 128, device=DEV)
    assert ix.dynakv_retrieve_attend_static(Q, 8, out, None) == binding.ECAPACITY
    assert spec.head_dim == 128
