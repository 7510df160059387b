"""Shared driver of the GPU parity tests: runs the HIP library and the CPU oracle on the same seeded
inputs, call by call, and compares them element by element.

Bars (from the benchmark spec): cluster memberships, selected-cluster sets and gather indices
bit-exact; centroids and attention outputs within 2e-3 relative (the library takes its integer
decisions on the same float64 quantities as the oracle, so centroids, M2 and tau are in fact compared
bit for bit); log-sum-exp within 2e-3 absolute.  Decisions whose margin is below 1e-4 are counted by the
oracle and reported, not excused.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import Oracle, OracleConfig
from paper_2511_07427_amd import binding
from paper_2511_07427_amd.workload import WorkloadSpec, generate

REL_TOL = 2e-3
LSE_TOL = 2e-3
DEV = "cuda:0"


def make_pair(spec: WorkloadSpec, n_units: int, max_tokens: int | None = None, **over):
    kw = dict(n_units=n_units, group_size=spec.group_size, n_clusters_init=spec.n_clusters_init,
              max_clusters=spec.max_clusters, max_tokens=max_tokens or spec.max_tokens, kmeans_iters=spec.kmeans_iters,
              buffer_max=spec.buffer_max, group_reduce=0, var_alpha=spec.var_alpha, size_factor=spec.size_factor,
              softmax_scale=0.0)
    kw.update(over)
    ix = binding.Index(binding.Config(dtype=spec.dtype, head_dim=spec.head_dim, **kw), DEV)
    o = Oracle(OracleConfig(head_dim=spec.head_dim, dtype=spec.dtype, **kw))
    return ix, o


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV).to(binding.TORCH_DTYPES[dtype]).contiguous()


def check_attention(out_g: np.ndarray, lse_g: np.ndarray, out_o: np.ndarray, lse_o: np.ndarray, what=""):
    """out: [U, G, d]; per (unit, head) vector: max |diff| / max(|oracle|_inf, 1e-6) <= REL_TOL."""
    den = np.maximum(np.abs(out_o).max(-1), 1e-6)
    rel = np.abs(out_g - out_o).max(-1) / den
    assert np.isfinite(out_g).all(), what
    assert rel.max() <= REL_TOL, "%s attention output off by %.3g (relative)" % (what, rel.max())
    fin = np.isfinite(lse_o)
    assert np.array_equal(np.isfinite(lse_g), fin), what
    if fin.any():
        err = np.abs(lse_g[fin] - lse_o[fin]).max()
        assert err <= LSE_TOL, "%s lse off by %.3g" % (what, err)
    return float(rel.max())


def _pairs(ix: binding.Index, units):
    """(unit of the library's index, unit of the oracle's): the oracle holds either all units or the sample `units`."""
    return list(enumerate(range(ix.cfg.n_units) if units is None else units))


def compare_retrieval(ix: binding.Index, o: Oracle, what="", gather=True, units=None):
    """Scores, selected clusters (ordered) and gather indices (ordered) of the last retrieval, bit for bit.
    The gather indices can only be read back before the next split (which may recycle the pages the gather
    list points to): after a whole-step call pass gather=False."""
    fields = ["n_selected", "selected", "n_gathered", "scores"] + (["gathered"] if gather else [])
    st = {k: v.numpy() for k, v in ix.dynakv_export_state(fields).items()}
    for ou, u in _pairs(ix, units):
        w = "%s unit %d" % (what, u)
        sel, gat, sc = o.selected(ou), o.gather(ou), o.scores(ou)
        assert st["n_selected"][u] == len(sel), w
        np.testing.assert_array_equal(st["selected"][u, :len(sel)], sel, err_msg=w + " selected clusters")
        assert st["n_gathered"][u] == len(gat), w
        if gather:
            np.testing.assert_array_equal(st["gathered"][u, :len(gat)], gat, err_msg=w + " gather indices")
        np.testing.assert_array_equal(st["scores"][u, :len(sc)], sc, err_msg=w + " scores")


def compare_state(ix: binding.Index, o: Oracle, what="", full=True, units=None):
    """Partition and per-cluster statistics of every unit, bit for bit."""
    fields = ["n_clusters", "n_tokens", "error", "size", "buffered", "flag", "last_assign"]
    if full:
        fields += ["tau", "centroids", "m2", "offsets", "members", "counters"]
    st = {k: v.numpy() for k, v in ix.dynakv_export_state(fields).items()}
    for ou, u in _pairs(ix, units):
        w = "%s unit %d" % (what, u)
        M, N = o.num_clusters(ou), o.num_tokens(ou)
        assert st["n_clusters"][u] == M and st["n_tokens"][u] == N, w
        assert st["error"][u] == o.error(ou), w
        c = o.clusters(ou)
        np.testing.assert_array_equal(st["size"][u, :M], c["n"], err_msg=w)
        np.testing.assert_array_equal(st["buffered"][u, :M], c["b"], err_msg=w)
        np.testing.assert_array_equal(st["flag"][u, :M], c["flag"], err_msg=w)
        assert st["last_assign"][u] == o.last_assign(ou), w
        if full:
            off, mem = o.members(ou)
            np.testing.assert_array_equal(st["offsets"][u, :M + 1], off, err_msg=w)
            np.testing.assert_array_equal(st["members"][u, :N], mem, err_msg=w + " memberships")
            np.testing.assert_array_equal(st["centroids"][u, :M], c["centroids"], err_msg=w + " centroids")
            np.testing.assert_array_equal(st["m2"][u, :M], c["M2"], err_msg=w + " M2")
            assert st["tau"][u] == o.tau(ou), w
            d = o.diagnostics(ou)
            assert (st["counters"][u, 0], st["counters"][u, 1], st["counters"][u, 2]) == \
                (d["splits"], d["failed_splits"], d["forced_splits"]), w
    return st


def run_trajectory(spec: WorkloadSpec, units, steps: int, budget: int | None = None, check_every: int = 1,
                   full_every: int = 64, step_call: str = "three", **over):
    """Builds both indexes on the given units of the workload and runs `steps` decode steps side by side.
    step_call: "three" = retrieve_attend, append, split; "one" = dynakv_decode_step; "mixed" = they alternate."""
    units = list(units)
    w = generate(spec, units=units, steps=steps)
    ix, o = make_pair(spec, len(units), max_tokens=spec.prefill + steps, **over)
    budget = spec.budget if budget is None else budget
    K0, V0 = to_dev(w["K0"], spec.dtype), to_dev(w["V0"], spec.dtype)
    init = torch.from_numpy(w["init_idx"]).to(DEV)
    ix.dynakv_build_index(K0, V0, init)
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    compare_state(ix, o, "after build_index")
    Qd, Kd, Vd = to_dev(w["Q"], spec.dtype), to_dev(w["Knew"], spec.dtype), to_dev(w["Vnew"], spec.dtype)
    U, G, d = len(units), spec.group_size, spec.head_dim
    out = torch.empty(U, G, d, dtype=torch.float32, device=DEV)
    lse = torch.empty(U, G, dtype=torch.float32, device=DEV)
    worst = 0.0
    most_splits = 0                    # largest number of splits of one unit in one step
    for t in range(steps):
        m_before = [o.num_clusters(u) for u in range(U)]
        whole = step_call == "one" or (step_call == "mixed" and t % 2 == 1)
        check = t % check_every == 0 or t == steps - 1
        oo, ol = o.retrieve_attend(w["Q"][t], budget)
        if whole:
            ix.dynakv_decode_step(Qd[t], budget, out, lse, Kd[t], Vd[t])
        else:
            ix.dynakv_retrieve_attend(Qd[t], budget, out, lse)
        if check:
            worst = max(worst, check_attention(out.cpu().numpy(), lse.cpu().numpy(), oo, ol, "step %d" % t))
            compare_retrieval(ix, o, "step %d" % t, gather=not whole)
        if not whole:
            ix.dynakv_append(Kd[t], Vd[t])
            ix.dynakv_split()
        o.append(w["Knew"][t], w["Vnew"][t])
        o.split()
        most_splits = max(most_splits, max(o.num_clusters(u) - m_before[u] for u in range(U)))
        if check:
            compare_state(ix, o, "step %d" % t, full=(t % full_every == 0 or t == steps - 1))
    diag = [o.diagnostics(u) for u in range(U)]
    return dict(worst_rel=worst, ties={k: sum(dd["ties"][k] for dd in diag) for k in diag[0]["ties"]},
                splits=sum(dd["splits"] for dd in diag), forced=sum(dd["forced_splits"] for dd in diag),
                clusters=[o.num_clusters(u) for u in range(U)], most_splits_in_a_step=most_splits,
                index=ix, oracle=o, workload=w)


def run_full_size(spec: WorkloadSpec, sample, steps: int, check_every: int = 16, full_every: int = 64):
    """The library on ALL units of the configuration, through the whole-step call and in its default launch
    shape (what the benchmark times), beside the oracle on the units `sample`: attention outputs, retrieval and
    index state of the sampled units are compared as in run_trajectory."""
    sample = list(sample)
    w = generate(spec, steps=steps, workers=16)
    kw = dict(group_size=spec.group_size, n_clusters_init=spec.n_clusters_init, max_clusters=spec.max_clusters,
              max_tokens=spec.prefill + steps, kmeans_iters=spec.kmeans_iters, buffer_max=spec.buffer_max, group_reduce=0,
              var_alpha=spec.var_alpha, size_factor=spec.size_factor, softmax_scale=0.0)
    ix = binding.Index(binding.Config(dtype=spec.dtype, head_dim=spec.head_dim, n_units=spec.n_units, **kw), DEV)
    o = Oracle(OracleConfig(head_dim=spec.head_dim, dtype=spec.dtype, n_units=len(sample), **kw))
    ix.dynakv_build_index(to_dev(w["K0"], spec.dtype), to_dev(w["V0"], spec.dtype), torch.from_numpy(w["init_idx"]).to(DEV))
    o.build_index(w["K0"][sample], w["V0"][sample], w["init_idx"][sample])
    compare_state(ix, o, "after build_index", units=sample)
    Qd, Kd, Vd = to_dev(w["Q"], spec.dtype), to_dev(w["Knew"], spec.dtype), to_dev(w["Vnew"], spec.dtype)
    out = torch.empty(spec.n_units, spec.group_size, spec.head_dim, dtype=torch.float32, device=DEV)
    lse = torch.empty(spec.n_units, spec.group_size, dtype=torch.float32, device=DEV)
    worst = 0.0
    for t in range(steps):
        check = t % check_every == 0 or t == steps - 1
        oo, ol = o.retrieve_attend(w["Q"][t][sample], spec.budget)
        ix.dynakv_decode_step(Qd[t], spec.budget, out, lse, Kd[t], Vd[t])
        if check:
            og, lg = out.cpu().numpy(), lse.cpu().numpy()
            assert np.isfinite(og).all(), "step %d" % t
            worst = max(worst, check_attention(og[sample], lg[sample], oo, ol, "step %d" % t))
            compare_retrieval(ix, o, "step %d" % t, gather=False, units=sample)
        o.append(w["Knew"][t][sample], w["Vnew"][t][sample])
        o.split()
        if check:
            compare_state(ix, o, "step %d" % t, full=(t % full_every == 0 or t == steps - 1), units=sample)
    err = ix.dynakv_export_state(["error"])["error"].numpy()
    assert not err.any(), "error words %s" % np.unique(err)
    diag = [o.diagnostics(k) for k in range(len(sample))]
    return dict(worst_rel=worst, splits=sum(dd["splits"] for dd in diag), forced=sum(dd["forced_splits"] for dd in diag),
                clusters=[o.num_clusters(k) for k in range(len(sample))])
