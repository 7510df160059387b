"""Shared driver of the GPU parity tests: runs the HIP library and the CPU oracle on the same seeded
inputs, call by call, and compares them.

Bars: cluster memberships, selected-cluster sets and gather indices bit-exact wherever
the oracle's margin for the decision exceeds 1e-4; centroids and attention outputs within 2e-3 relative, M2 and
tau within 2e-3 relative, log-sum-exp within 2e-3 absolute (plus 2^-17 of its magnitude, the float32 accumulation
bound, which only matters for logits of the order of 10^4).  A disagreement on a decision whose margin is at
most 1e-4 is a tie: it is counted per class (assign, trigger, select, split), printed by the tests, and the
oracle's unit is then re-synchronised from the library's exported state (dynakv_export_state ->
Oracle.import_unit) so that the run can go on side by side.  A disagreement above the margin fails.
Every decision is compared at every step; attention outputs and the full state at the given intervals.
"""
from __future__ import annotations

from collections import Counter

import numpy as np
import torch

from oracle import Oracle, OracleConfig
from paper_2511_07427_amd import binding
from paper_2511_07427_amd.workload import WorkloadSpec, generate

REL_TOL = 2e-3
LSE_TOL = 2e-3
MARGIN = 1e-4
DEV = "cuda:0"


def make_pair(spec: WorkloadSpec, n_units: int, max_tokens: int | None = None, oracle_units: int | None = None, **over):
    kw = dict(group_size=spec.group_size, n_clusters_init=spec.n_clusters_init,
              max_clusters=spec.max_clusters, max_tokens=max_tokens or spec.max_tokens, kmeans_iters=spec.kmeans_iters,
              buffer_max=spec.buffer_max, group_reduce=0, var_alpha=spec.var_alpha, size_factor=spec.size_factor,
              softmax_scale=0.0, search_copy=0, score_round=0, update_mode=0)
    launch = over.pop("launch", 0)
    kw.update(over)
    ix = binding.Index(binding.Config(dtype=spec.dtype, head_dim=spec.head_dim, n_units=n_units, launch=launch, **kw), DEV)
    if spec.dtype == "f32":
        kw["search_copy"] = 1            # float32 storage: the search copy is the mean itself on both sides
    o = Oracle(OracleConfig(head_dim=spec.head_dim, dtype=spec.dtype, n_units=oracle_units or n_units, **kw))
    return ix, o


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV).to(binding.TORCH_DTYPES[dtype]).contiguous()


def check_attention(out_g: np.ndarray, lse_g: np.ndarray, out_o: np.ndarray, lse_o: np.ndarray, what=""):
    """out: [U, G, d]; per (unit, head) vector: max |diff| / max(|oracle|_inf, 1e-6) <= REL_TOL."""
    if out_g.shape[0] == 0:
        return 0.0
    den = np.maximum(np.abs(out_o).max(-1), 1e-6)
    rel = np.abs(out_g - out_o).max(-1) / den
    assert np.isfinite(out_g).all(), what
    assert rel.max() <= REL_TOL, "%s attention output off by %.3g (relative)" % (what, rel.max())
    fin = np.isfinite(lse_o)
    assert np.array_equal(np.isfinite(lse_g), fin), what
    if fin.any():
        # 2e-3 absolute, plus what float32 can hold at the value's magnitude: the logits are 128 exact products
        # accumulated in float32 (relative error up to 128 * 2^-24 = 2^-17), and keys that have drifted far make
        # logits, and with them the log-sum-exp, of the order of 10^4
        err = np.abs(lse_g[fin] - lse_o[fin]) - 2.0 ** -17 * np.abs(lse_o[fin])
        assert err.max() <= LSE_TOL, "%s lse off by %.3g" % (what, np.abs(lse_g[fin] - lse_o[fin]).max())
    return float(rel.max())


def _pairs(ix: binding.Index, units):
    """(unit of the oracle's index, unit of the library's): the oracle holds either all units or the sample `units`."""
    return list(enumerate(range(ix.cfg.n_units) if units is None else units))


def score_bound(ix: binding.Index, Q: np.ndarray, centroids: np.ndarray) -> float:
    """Largest difference allowed between a score of the library and the oracle's: the library accumulates the
    128 exact products of a score in float32 on the matrix cores (error at most 128 * 2^-24 * |q| |r|, doubled
    here), and both round the scaled result to float32 or not."""
    scale = ix.cfg.softmax_scale or 1.0 / np.sqrt(ix.cfg.head_dim)
    qn = np.sqrt((Q.astype(np.float64) ** 2).sum(-1)).max() * (ix.cfg.group_size if ix.cfg.group_reduce else 1)
    rn = np.sqrt((centroids.astype(np.float64) ** 2).sum(-1)).max()
    return 2.0 ** -16 * scale * qn * rn * 1.01 + 1e-30


class Tally(Counter):
    """Ties by class, re-synchronisations, worst value errors; `offsets`: per oracle unit, the library's split
    counters minus the oracle's at the last re-synchronisation (after a tie the two have counted different events)."""

    def __init__(self):
        super().__init__()
        self.offsets = {}

    def worst(self, key, val):
        self[key] = max(self.get(key, 0.0), float(val))


def resync(ix: binding.Index, o: Oracle, units, dirty, tally: Tally):
    """The oracle's units `dirty` (oracle numbering) take the library's exported state."""
    if not dirty:
        return
    pairs = [(ou, u) for ou, u in _pairs(ix, units) if ou in dirty]
    dev = ix.dynakv_export_state(binding.IMPORT_FIELDS + ("counters",), to_cpu=False)
    idx = torch.tensor([u for _, u in pairs], device=DEV)
    st = {k: v.index_select(0, idx).cpu() for k, v in dev.items()}      # only the units that are taken cross the bus
    del dev
    for u, (ou, _) in enumerate(pairs):
        M, N, ns = int(st["n_clusters"][u]), int(st["n_tokens"][u]), int(st["n_selected"][u])
        o.import_unit(ou, st["keys"][u, :N].float().numpy(), st["values"][u, :N].float().numpy(),
                      st["centroids"][u, :M].numpy(), st["size"][u, :M].numpy(), st["buffered"][u, :M].numpy(),
                      st["flag"][u, :M].numpy(), st["m2"][u, :M].numpy(), st["offsets"][u, :M + 1].numpy(),
                      st["members"][u, :N].numpy(), float(st["tau"][u]), st["selected"][u, :ns].numpy())
        d = o.diagnostics(ou)
        tally.offsets[ou] = st["counters"][u, :3].numpy() - np.array([d["splits"], d["failed_splits"], d["forced_splits"]])


def compare_retrieval(ix: binding.Index, o: Oracle, tally: Tally, what="", gather=True, units=None, Q=None, budget=None,
                      skip=()):
    """Scores, selected set, order and gather indices of the last retrieval.  Returns the oracle units whose
    selection differs by a tie.  The gather indices can only be read back before the next split (which may
    recycle the pages the gather list points to): after a whole-step call pass gather=False."""
    fields = ["n_selected", "selected", "n_gathered", "scores", "n_clusters"] + (["gathered"] if gather else [])
    st = {k: v.numpy() for k, v in ix.dynakv_export_state(fields).items()}
    dirty = set()
    for ou, u in _pairs(ix, units):
        if ou in skip:
            continue
        w = "%s unit %d" % (what, u)
        sel, gat, sc = o.selected(ou), o.gather(ou), o.scores(ou)
        M = min(len(sc), int(st["n_clusters"][u]))      # (a local clustering after the retrieval leaves fewer clusters)
        sc_all, sc = sc, sc[:M]
        if Q is not None:
            tol = score_bound(ix, Q[ou], o.search_copy(ou))
            err = np.abs(st["scores"][u, :M].astype(np.float64) - sc).max()
            tally.worst("score_err_over_bound", err / tol)
            assert err <= tol + 6e-8 * max(1.0, np.abs(sc).max()), "%s scores off by %.3g (bound %.3g)" % (w, err, tol)
        gsel = st["selected"][u, :st["n_selected"][u]]
        if set(gsel.tolist()) != set(sel.tolist()) or st["n_gathered"][u] != len(gat):
            mg = o.diagnostics(ou)["margin_select"]
            assert mg <= MARGIN, "%s selected sets differ at margin %.3g: library %s, oracle %s" % (
                w, mg, sorted(set(gsel.tolist()) - set(sel.tolist())), sorted(set(sel.tolist()) - set(gsel.tolist())))
            tally["tie_select"] += 1
            dirty.add(ou)
            continue
        # same set.  The order in which the clusters are attended is the library's own: ascending id, or, where the
        # selection keeps its keys in memory (more than 16384 clusters), the oracle's score order up to the bound
        if len(gsel) > 1 and not (np.diff(gsel) > 0).all():
            s_in_order = sc_all[gsel]
            slack = (score_bound(ix, Q[ou], o.search_copy(ou)) if Q is not None else 0.0) * 2 + 1.2e-7 * np.abs(s_in_order).max()
            worst = (s_in_order[1:] - s_in_order[:-1]).max()
            assert worst <= slack, "%s selected clusters out of score order by %.3g" % (w, worst)
        if gather:
            off, mem = o.members(ou)
            want = np.concatenate([mem[off[j]:off[j + 1]] for j in gsel]) if len(gsel) else np.zeros(0, np.int32)
            if budget is not None and len(want) > len(gat):       # the best cluster alone is over budget: cut to it
                want = want[:budget]
            np.testing.assert_array_equal(st["gathered"][u, :len(want)], want, err_msg=w + " gather indices")
            assert sorted(want.tolist()) == sorted(gat.tolist()), w + " gathered entries"
    return dirty


def _rel(a, b, floor):
    return np.abs(a - b) / np.maximum(np.abs(b), floor)


def compare_state(ix: binding.Index, o: Oracle, tally: Tally, what="", full=True, units=None, skip=(), assign=True):
    """Partition and per-cluster statistics.  Returns the oracle units that differ from the library by a tie
    (their comparison stops at the decision that differs)."""
    fields = ["n_clusters", "n_tokens", "error", "size", "buffered", "flag", "last_assign"]
    if full:
        fields += ["tau", "centroids", "m2", "offsets", "members", "counters"]
    st = {k: v.numpy() for k, v in ix.dynakv_export_state(fields).items()}
    dirty = set()
    for ou, u in _pairs(ix, units):
        if ou in skip:
            continue
        w = "%s unit %d" % (what, u)
        M, N = o.num_clusters(ou), o.num_tokens(ou)
        c, d = o.clusters(ou), o.diagnostics(ou)
        assert st["n_tokens"][u] == N and st["error"][u] == o.error(ou), w
        # the step's decisions in the order they were taken: nearest cluster, threshold test, splits
        if assign and st["last_assign"][u] != o.last_assign(ou):
            assert d["margin_assign"] <= MARGIN, "%s nearest cluster %d vs %d at margin %.3g" % (
                w, st["last_assign"][u], o.last_assign(ou), d["margin_assign"])
            tally["tie_assign"] += 1
            dirty.add(ou)
            continue
        same_shape = st["n_clusters"][u] == M
        eq = same_shape and all(np.array_equal(st[k][u, :M], c[n]) for k, n in (("size", "n"), ("buffered", "b"), ("flag", "flag")))
        if eq and full:
            off, mem = o.members(ou)
            eq = np.array_equal(st["offsets"][u, :M + 1], off) and np.array_equal(st["members"][u, :N], mem)
        if not eq:
            ja = o.last_assign(ou)
            only_trigger = same_shape and d["margin_trigger"] <= MARGIN and all(
                np.array_equal(np.delete(st[k][u, :M], ja), np.delete(c[n], ja)) for k, n in (("size", "n"), ("buffered", "b"), ("flag", "flag")))
            if only_trigger:
                tally["tie_trigger"] += 1
            else:
                assert d["margin_split"] <= MARGIN or d["margin_trigger"] <= MARGIN, \
                    "%s partitions differ (clusters %d vs %d) at margins trigger %.3g split %.3g" % (
                        w, st["n_clusters"][u], M, d["margin_trigger"], d["margin_split"])
                tally["tie_split" if d["margin_split"] <= MARGIN else "tie_trigger"] += 1
            dirty.add(ou)
            continue
        if full:
            den = np.maximum(np.abs(c["centroids"]).max(-1), 1e-6)
            cerr = (np.abs(st["centroids"][u, :M] - c["centroids"]).max(-1) / den).max()
            merr = _rel(st["m2"][u, :M], c["M2"], 1e-6).max()
            terr = abs(st["tau"][u] - o.tau(ou)) / max(abs(o.tau(ou)), 1e-6)
            tally.worst("centroid_rel", cerr); tally.worst("m2_rel", merr); tally.worst("tau_rel", terr)
            assert cerr <= REL_TOL, "%s centroids off by %.3g" % (w, cerr)
            assert merr <= REL_TOL, "%s M2 off by %.3g" % (w, merr)
            assert terr <= REL_TOL, "%s tau off by %.3g" % (w, terr)
            cnt = st["counters"][u, :3] - tally.offsets.get(ou, 0)
            assert tuple(cnt) == (d["splits"], d["failed_splits"], d["forced_splits"]), "%s split counters %s vs %s" % (w, cnt, d)
    return dirty


def compare_build(ix: binding.Index, o: Oracle, tally: Tally, n0: int, units=None):
    """After build_index: labels must be equal wherever the k-means margin of the point exceeds 1e-4 in every
    iteration; one point below it decides differently and the centres after it legitimately differ, so such a
    unit is counted as a tie and re-synchronised."""
    st = {k: v.numpy() for k, v in ix.dynakv_export_state(["n_clusters", "offsets", "members", "error"]).items()}
    dirty = set()
    for ou, u in _pairs(ix, units):
        M = o.num_clusters(ou)
        off, mem = o.members(ou)
        assert st["n_clusters"][u] == M and st["error"][u] == 0
        if not (np.array_equal(st["offsets"][u, :M + 1], off) and np.array_equal(st["members"][u, :n0], mem)):
            assert o.kmeans_margins(ou, n0).min() <= MARGIN, "k-means labels differ, unit %d, no point within the margin" % u
            tally["tie_kmeans"] += 1
            dirty.add(ou)
    resync(ix, o, units, dirty, tally)
    d2 = compare_state(ix, o, tally, "after build_index", units=units)
    assert not d2


class Stepper:
    """Drives both sides through decode steps and applies the protocol above."""

    def __init__(self, ix, o, spec, w, units=None, budget=None):
        self.ix, self.o, self.spec, self.w, self.units = ix, o, spec, w, units
        self.budget = spec.budget if budget is None else budget
        self.tally = Tally()
        U, G, d = ix.cfg.n_units, spec.group_size, spec.head_dim
        self.out = torch.empty(U, G, d, dtype=torch.float32, device=DEV)
        self.lse = torch.empty(U, G, dtype=torch.float32, device=DEV)
        self.Qd, self.Kd, self.Vd = (to_dev(w[k], spec.dtype) for k in ("Q", "Knew", "Vnew"))
        self.sel = slice(None) if units is None else list(units)
        self.worst = 0.0
        self.most_splits = 0

    def step(self, t, whole: bool, attention: bool, full: bool):
        ix, o, w, tally = self.ix, self.o, self.w, self.tally
        Q = w["Q"][t][self.sel]
        nu = Q.shape[0]
        m_before = [o.num_clusters(k) for k in range(nu)]
        oo, ol = o.retrieve_attend(Q, self.budget)
        if whole:
            ix.dynakv_decode_step(self.Qd[t], self.budget, self.out, self.lse, self.Kd[t], self.Vd[t])
        else:
            ix.dynakv_retrieve_attend(self.Qd[t], self.budget, self.out, self.lse)
        dirty = compare_retrieval(ix, o, tally, "step %d" % t, gather=not whole, units=self.units, Q=Q, budget=self.budget)
        if attention:
            og, lg = self.out.cpu().numpy(), self.lse.cpu().numpy()
            assert np.isfinite(og).all(), "step %d" % t
            keep = [k for k in range(nu) if k not in dirty]
            gk = [self.sel[k] for k in keep] if self.units is not None else keep
            self.worst = max(self.worst, check_attention(og[gk], lg[gk], oo[keep], ol[keep], "step %d" % t))
        if not whole:
            ix.dynakv_append(self.Kd[t], self.Vd[t])
            ix.dynakv_split()
        o.append(w["Knew"][t][self.sel], w["Vnew"][t][self.sel])
        o.split()
        self.most_splits = max(self.most_splits, max(o.num_clusters(k) - m_before[k] for k in range(nu)))
        dirty |= compare_state(ix, o, tally, "step %d" % t, full=full, units=self.units, skip=dirty)
        if dirty:
            tally["resyncs"] += len(dirty)
            resync(ix, o, self.units, dirty, tally)

    def report(self):
        o = self.o
        nu = len(self.sel) if self.units is not None else self.ix.cfg.n_units
        diag = [o.diagnostics(k) for k in range(nu)]
        return dict(worst_rel=self.worst, ties=dict(self.tally),
                    oracle_low_margin={k: sum(dd["ties"][k] for dd in diag) for k in diag[0]["ties"]},
                    splits=sum(dd["splits"] for dd in diag), forced=sum(dd["forced_splits"] for dd in diag),
                    failed=sum(dd["failed_splits"] for dd in diag),
                    clusters=[o.num_clusters(k) for k in range(nu)], most_splits_in_a_step=self.most_splits)


def run_trajectory(spec: WorkloadSpec, units, steps: int, budget: int | None = None, check_every: int = 1,
                   full_every: int = 64, step_call: str = "three", **over):
    """Builds both indexes on the given units of the workload and runs `steps` decode steps side by side.
    step_call: "three" = retrieve_attend, append, split; "one" = dynakv_decode_step; "mixed" = they alternate."""
    units = list(units)
    w = generate(spec, units=units, steps=steps)
    ix, o = make_pair(spec, len(units), max_tokens=spec.prefill + steps, **over)
    K0, V0 = to_dev(w["K0"], spec.dtype), to_dev(w["V0"], spec.dtype)
    init = torch.from_numpy(w["init_idx"]).to(DEV)
    ix.dynakv_build_index(K0, V0, init)
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    s = Stepper(ix, o, spec, w, None, budget)
    compare_build(ix, o, s.tally, spec.prefill)
    for t in range(steps):
        whole = step_call == "one" or (step_call == "mixed" and t % 2 == 1)
        s.step(t, whole, attention=(t % check_every == 0 or t == steps - 1), full=(t % full_every == 0 or t == steps - 1))
    r = s.report()
    r.update(index=ix, oracle=o, workload=w)
    return r


def run_full_size(spec: WorkloadSpec, sample, steps: int, check_every: int = 16, full_every: int = 64, **over):
    """The library on ALL units of the configuration, through the whole-step call and in its default launch
    shape (what the benchmark times), beside the oracle on the units `sample`: attention outputs, retrieval and
    index state of the sampled units are compared as in run_trajectory."""
    sample = list(sample)
    w = generate(spec, steps=steps, workers=16)
    ix, o = make_pair(spec, spec.n_units, max_tokens=spec.prefill + steps, oracle_units=len(sample), **over)
    ix.dynakv_build_index(to_dev(w["K0"], spec.dtype), to_dev(w["V0"], spec.dtype), torch.from_numpy(w["init_idx"]).to(DEV))
    o.build_index(w["K0"][sample], w["V0"][sample], w["init_idx"][sample])
    s = Stepper(ix, o, spec, w, sample)
    compare_build(ix, o, s.tally, spec.prefill, units=sample)
    for t in range(steps):
        s.step(t, True, attention=(t % check_every == 0 or t == steps - 1), full=(t % full_every == 0 or t == steps - 1))
    err = ix.dynakv_export_state(["error"])["error"].numpy()
    assert not err.any() and ix.export_status == binding.OK, "error words %s" % np.unique(err)
    return s.report()


def run_window(spec: WorkloadSpec, sample, start: int, steps: int, check_every: int = 8, **over):
    """Late-state parity: the library alone runs ALL units of the configuration from prefill to step `start`
    (whole-step calls, nothing compared); its state is then exported, the oracle imports the units `sample`, and
    both run `steps` more steps side by side under the protocol above.  The workload is generated once for
    start + steps steps, so the window is the one a run of that length reaches."""
    sample = list(sample)
    T = start + steps
    w = generate(spec, steps=T, workers=16)
    ix, o = make_pair(spec, spec.n_units, max_tokens=spec.prefill + T, oracle_units=len(sample), **over)
    ix.dynakv_build_index(to_dev(w["K0"], spec.dtype), to_dev(w["V0"], spec.dtype), torch.from_numpy(w["init_idx"]).to(DEV))
    s = Stepper(ix, o, spec, w, sample)
    for t in range(start):
        ix.dynakv_decode_step(s.Qd[t], s.budget, s.out, s.lse, s.Kd[t], s.Vd[t])
    err = ix.dynakv_export_state(["error"])["error"].numpy()
    assert not err.any(), "error words %s before the window" % np.unique(err)
    resync(ix, o, sample, set(range(len(sample))), s.tally)
    d0 = compare_state(ix, o, s.tally, "imported state", units=sample, assign=False)
    assert not d0
    for t in range(start, T):
        s.step(t, True, attention=((t - start) % check_every == 0 or t == T - 1), full=(t == T - 1))
    err = ix.dynakv_export_state(["error"])["error"].numpy()
    assert not err.any() and ix.export_status == binding.OK, "error words %s" % np.unique(err)
    return s.report()
