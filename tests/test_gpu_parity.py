"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs.

Sizes are chosen so the oracle finishes in seconds while every kernel still sees several tiles, ragged
tails and (where the workload drifts) real splits.  Each of the five benchmark configurations appears
with its own storage type, group size, cluster count and budget, on a few of its units.
"""
import json
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import parity  # noqa: E402
from parity import DEV, Tally, check_attention, compare_build, compare_retrieval, compare_state, make_pair, run_trajectory, to_dev  # noqa: E402
from paper_2511_07427_amd import binding  # noqa: E402
from paper_2511_07427_amd.binding import LAUNCH_SEPARATE, LAUNCH_SPLIT_KERNEL, launch_shape  # noqa: E402
from paper_2511_07427_amd.workload import CONFIGS, WorkloadSpec, generate  # noqa: E402

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def say(*a):
    print(*a, flush=True)


# --------------------------------------------------------------------------- the five configurations

def test_cfg1_tiny_f32_full_trajectory():
    s = CONFIGS["tiny"]
    r = run_trajectory(s, [0], s.steps, check_every=1, full_every=16)
    say("tiny:", {k: r[k] for k in ("worst_rel", "ties", "oracle_low_margin", "splits", "clusters")})
    assert r["splits"] > 0


def test_cfg1_tiny_with_variance_trigger_and_small_buffer():
    s = CONFIGS["tiny"].scaled(var_alpha=1.2, buffer_max=4)
    r = run_trajectory(s, [0], s.steps, budget=128, check_every=1, full_every=16)
    say("tiny/var:", {k: r[k] for k in ("worst_rel", "ties", "splits", "forced", "clusters")})
    assert r["splits"] > 0 and r["forced"] > 0


def test_cfg2_llama_shaped_f16():
    s = CONFIGS["llama3_8b"]
    r = run_trajectory(s, [0, 17, 255], 384, check_every=4, full_every=64)
    say("llama:", {k: r[k] for k in ("worst_rel", "ties", "splits", "forced", "clusters")})


def test_cfg3_qwen_shaped_bf16_group_of_7():
    s = CONFIGS["qwen25_7b"]
    r = run_trajectory(s, [0, 111], 768, check_every=8, full_every=128)
    say("qwen:", {k: r[k] for k in ("worst_rel", "ties", "splits", "forced", "clusters")})
    assert r["splits"] > 0


def test_cfg4_batched_shaped_f16():
    s = CONFIGS["batched16"]
    r = run_trajectory(s, [3, 64], 128, check_every=4, full_every=64)
    say("batched:", {k: r[k] for k in ("worst_rel", "ties", "splits", "forced", "clusters")})


def test_cfg5_long_shaped_bf16_group_of_8():
    s = CONFIGS["long131k"].scaled(kmeans_iters=3)
    r = run_trajectory(s, [5], 192, check_every=8, full_every=96)
    say("long:", {k: r[k] for k in ("worst_rel", "ties", "splits", "forced", "clusters")})


# --------------------------------------------------------------------------- launch shapes of the retrieval

@pytest.mark.parametrize("name,units,steps,launch", [
    ("llama3_8b", [1, 2], 96, launch_shape(1)),                          # one kernel per retrieval, G = 4
    ("qwen25_7b", [3], 160, launch_shape(1)),                            # one kernel per retrieval, G = 7
    ("llama3_8b", [4], 64, launch_shape(1, 0, LAUNCH_SEPARATE)),         # separate kernels, no split-KV
    ("long131k", [2], 48, launch_shape(3, 8)),                           # split-KV with prefetching wavefronts
    ("llama3_8b", [5, 6], 64, launch_shape(5, 16, LAUNCH_SEPARATE)),     # split-KV, 16 wavefronts, odd split count
])
def test_every_launch_shape_of_retrieve_attend(name, units, steps, launch):
    s = CONFIGS[name]
    if name == "long131k":
        s = s.scaled(kmeans_iters=2)
    if name == "llama3_8b":
        s = s.scaled(max_cluster_factor=8)
    r = run_trajectory(s, units, steps, check_every=1, full_every=32, step_call="mixed", launch=launch)
    say(name, hex(launch), {k: r[k] for k in ("worst_rel", "ties", "splits", "clusters")})


@pytest.mark.parametrize("name,units,steps,launch", [
    ("llama3_8b", [7, 8, 9], 160, launch_shape(1)),                        # the whole step in one kernel, G = 4
    ("qwen25_7b", [5, 6], 256, launch_shape(1)),                           # the same with G = 7
    ("llama3_8b", [7, 8, 9], 160, launch_shape(1, 0, LAUNCH_SPLIT_KERNEL)),   # retrieval + append in one kernel, splits in their own
    ("batched16", [9], 64, launch_shape(0, 0, LAUNCH_SEPARATE)),           # separate kernels behind the same call
])
def test_whole_step_call_matches_the_three_calls(name, units, steps, launch):
    s = CONFIGS[name]
    r = run_trajectory(s, units, steps, check_every=1, full_every=32, step_call="one", launch=launch)
    say(name, hex(launch), {k: r[k] for k in ("worst_rel", "ties", "splits", "forced", "clusters")})
    assert r["splits"] > 0 or name == "batched16"


def test_long_run_through_the_whole_step_call_with_several_splits_per_step():
    # the steady state of the benchmark configuration in its launch shape (one workgroup per unit, the whole
    # step in one kernel): small clusters, several due splits of one unit in one step (decided by separate
    # wavefronts while the pages are streamed, the fourth after the attention)
    s = CONFIGS["llama3_8b"]
    r = run_trajectory(s, [16, 17, 18, 19, 20, 21, 22, 23], 2560, check_every=32, full_every=640, step_call="one",
                       launch=launch_shape(1))
    say("long:", {k: r[k] for k in ("worst_rel", "ties", "splits", "forced", "clusters", "most_splits_in_a_step")})
    assert r["splits"] > 2000 and r["most_splits_in_a_step"] >= 3


def test_long_run_through_the_whole_step_call_group_of_7():
    # the same for the kernel variant that holds up to 8 query heads per KV head (bf16, G = 7)
    s = CONFIGS["qwen25_7b"]
    r = run_trajectory(s, [30, 31, 32, 33], 2048, check_every=32, full_every=512, step_call="one", launch=launch_shape(1))
    say("long, G = 7:", {k: r[k] for k in ("worst_rel", "ties", "splits", "forced", "clusters", "most_splits_in_a_step")})
    assert r["splits"] > 500 and r["most_splits_in_a_step"] >= 2


@pytest.mark.parametrize("dtype,step_call", [("f16", "one"), ("bf16", "one"), ("f32", "three"), ("f16", "three")])
def test_splits_of_large_clusters(dtype, step_call):
    # prefill clusters of several dozen to a few hundred entries that the drift splits early: up to 64 entries of a
    # 16-bit type (32 of float32) one wavefront each, four side by side; up to 128 (64) one wavefront each, two
    # side by side; larger ones by the whole workgroup.  The sizes of the clusters that were split are taken from
    # the oracle's records before and after every step.
    s = CONFIGS["llama3_8b"].scaled(dtype=dtype, prefill=1536, n_clusters_init=20, var_alpha=1.02, max_cluster_factor=16,
                                    kmeans_iters=4, budget=512)
    units, steps = [0, 1, 2, 3], 192
    w = generate(s, units=units, steps=steps)
    ix, o = make_pair(s, len(units), max_tokens=s.prefill + steps)
    ix.dynakv_build_index(to_dev(w["K0"], s.dtype), to_dev(w["V0"], s.dtype), torch.from_numpy(w["init_idx"]).to(DEV))
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    st = parity.Stepper(ix, o, s, w, None, None)
    compare_build(ix, o, st.tally, s.prefill)
    parents = []
    for t in range(steps):
        before = [o.clusters(k) for k in range(len(units))]
        st.step(t, step_call == "one", attention=t % 4 == 0, full=t % 32 == 0 or t == steps - 1)
        for k in range(len(units)):
            after = o.clusters(k)
            if len(after["n"]) > len(before[k]["n"]):
                m0 = before[k]["n"] + before[k]["b"]
                m1 = (after["n"] + after["b"])[:len(m0)]
                parents += [int(x) for x in m0[m1 < m0]]
    r = st.report()
    small = 32 if dtype == "f32" else 64
    hist = dict(one_per_lane=sum(p <= small for p in parents), two_per_lane=sum(small < p <= 2 * small for p in parents),
                workgroup=sum(p > 2 * small for p in parents))
    say("large clusters,", dtype, step_call, hist, {k: r[k] for k in ("worst_rel", "ties", "splits", "forced", "clusters")})
    assert hist["two_per_lane"] >= 3 and hist["workgroup"] >= 1 and (hist["one_per_lane"] >= 3 or dtype == "f32")


@pytest.mark.parametrize("dtype,step_call", [("f16", "one"), ("bf16", "one"), ("f16", "three"), ("f32", "three")])
def test_splits_of_degenerate_large_clusters(dtype, step_call):
    # one large cluster per unit that the size trigger flags at the first append and that is split at once
    # (B_max = 0): 100 equal keys (no second seed: unflagged with exact statistics), 99 equal keys and one apart
    # (split 99 / 1, the second seed is the lowest of 99 equally far members), two values of 60 keys each, and 129
    # equal keys (workgroup path)
    N0, d = 160, 128
    s = WorkloadSpec("degenerate", dtype, 4, 2, N0, 2, 2, 64, 6, 0.05, var_alpha=0.0, size_factor=1.0, buffer_max=0,
                     kmeans_iters=2, max_cluster_factor=8, seed=77)
    w = generate(s, steps=2)
    a = np.full(d, 5.0, np.float32)
    apart = a.copy(); apart[0] = 8.0
    b = a.copy(); b[:4] += 0.5
    K0 = w["K0"].copy()
    sizes = (100, 100, 120, 129)
    K0[0, :100] = a
    K0[1, :100] = a; K0[1, 57] = apart
    K0[2, :120:2] = a; K0[2, 1:120:2] = b
    K0[3, :129] = a
    init = np.array([[0, n] for n in sizes], np.int32)
    w = dict(w, K0=K0, init_idx=init)
    w["Knew"] = w["Knew"].copy(); w["Knew"][0, :] = a
    ix, o = make_pair(s, 4, max_tokens=N0 + 2)
    ix.dynakv_build_index(to_dev(K0, dtype), to_dev(w["V0"], dtype), torch.from_numpy(init).to(DEV))
    o.build_index(K0, w["V0"], init)
    st = parity.Stepper(ix, o, s, w, None, None)
    compare_build(ix, o, st.tally, N0)
    assert [int(o.clusters(k)["n"][0]) for k in range(4)] == list(sizes)
    for t in range(2):
        st.step(t, step_call == "one", attention=True, full=True)
    r = st.report()
    say("degenerate clusters,", dtype, step_call, {k: r[k] for k in ("worst_rel", "ties", "splits", "failed", "clusters")})
    assert r["failed"] == 2 and r["splits"] >= 2
    c1, c2 = o.clusters(1), o.clusters(2)
    assert {1, 100} <= set(c1["n"].tolist()) and {60, 61} <= set(c2["n"].tolist())


@pytest.mark.parametrize("name,sample,steps,iters", [
    ("llama3_8b", [0, 131, 255], 1280, None),     # what the benchmark times
    ("llama3_8b", [0, 100, 255], 8256, None),     # ... over its whole horizon (warm-up and timed steps)
    ("batched16", [0, 77, 127], 96, None),
    ("qwen25_7b", [0, 58, 111], 512, None),
    ("long131k", [6], 96, 3),                     # separate kernels, 4 workgroups per unit in gather + attention
])
def test_full_size_configurations_on_sampled_units(name, sample, steps, iters):
    # all units of the configuration, default launch shape, one whole-step call per step; the oracle follows
    # a few of the units (k-means shortened where the oracle's prefill would take minutes)
    s = CONFIGS[name] if iters is None else CONFIGS[name].scaled(kmeans_iters=iters)
    r = parity.run_full_size(s, sample, steps, check_every=32 if steps < 4096 else 64, full_every=256 if steps < 4096 else 512)
    say("full size, %s:" % name, r)
    assert r["splits"] > 0 or name in ("batched16", "long131k")


# --------------------------------------------------------------------------- late windows of the full horizons

@pytest.mark.parametrize("name,sample,start,steps", [
    ("batched16", [0, 77, 127], 24576 - 64, 64),     # the end of the window the configuration times (128 units, ~7200 clusters each)
    ("qwen25_7b", [0, 58, 111], 30000 - 64, 64),     # 112 units, ~12000 clusters each
    ("long131k", [0, 5], 114688 - 48, 48),           # 8 units, 131 072 entries each
])
def test_late_window_of_the_full_horizon(name, sample, start, steps):
    """All units of the configuration run alone from prefill to `start` (whole-step calls, the launch shape the
    benchmark times, cluster capacity for the full horizon); the state is then exported, the oracle imports the
    sampled units, and the last steps of the horizon run side by side under the parity protocol."""
    from paper_2511_07427_amd.workload import FULL_HORIZON_FACTOR
    s = CONFIGS[name].scaled(max_cluster_factor=FULL_HORIZON_FACTOR[name])
    r = parity.run_window(s, sample, start, steps, check_every=8)
    say("late window, %s:" % name, r)
    assert r["splits"] > 0 and min(r["clusters"]) > 4 * s.n_clusters_init


# --------------------------------------------------------------------------- hand-worked fixtures, padded to d = 128

def _pad(a):
    a = np.asarray(a, np.float32)
    out = np.zeros(a.shape[:-1] + (128,), np.float32)
    out[..., :a.shape[-1]] = a
    return out


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_hand_examples_on_the_gpu(dtype):
    g1 = json.load(open(os.path.join(GOLD, "hand_example_1_retrieve.json")))
    g3 = json.load(open(os.path.join(GOLD, "hand_example_3_split.json")))
    tdt = binding.TORCH_DTYPES[dtype]
    scale = float(1 / np.sqrt(2))
    # example 1: build, score, select, attend
    cfg = binding.Config(1, 1, dtype, 2, 8, 64, kmeans_iters=3, softmax_scale=scale)
    ix = binding.Index(cfg, DEV)
    K = torch.from_numpy(_pad(g1["keys"]))[None].to(DEV).to(tdt)
    V = torch.from_numpy(_pad(g1["values"]))[None].to(DEV).to(tdt)
    ix.dynakv_build_index(K, V, torch.tensor([g1["init_idx"]], dtype=torch.int32, device=DEV))
    st = ix.dynakv_export_state()
    assert st["size"][0, :2].tolist() == g1["clusters"]["n"]
    np.testing.assert_allclose(st["centroids"][0, :2, :2].numpy(), np.array(g1["clusters"]["centroids"], np.float32), rtol=1e-6)
    np.testing.assert_allclose(st["m2"][0, :2].numpy(), g1["clusters"]["M2"], rtol=1e-6)
    assert st["members"][0, :6].tolist() == sum(g1["clusters"]["members"], [])
    q = torch.from_numpy(_pad([[g1["query"]]])).to(DEV).to(tdt)
    out = torch.empty(1, 1, 128, device=DEV)
    lse = torch.empty(1, 1, device=DEV)
    ix.dynakv_retrieve_attend(q, 2, out, lse)
    st = ix.dynakv_export_state(binding._STATE_FIELDS)
    assert st["selected"][0, :st["n_selected"][0]].tolist() == g1["budget_2"]["selected"]
    assert st["gathered"][0, :st["n_gathered"][0]].tolist() == g1["budget_2"]["gather"]
    np.testing.assert_allclose(st["scores"][0, :2].numpy(), g1["scores"], rtol=1e-6)
    np.testing.assert_array_equal(st["keys"][0, :6].float().numpy(), _pad(g1["keys"]))
    np.testing.assert_array_equal(st["values"][0, :6].float().numpy(), _pad(g1["values"]))
    np.testing.assert_allclose(out[0, 0, :2].cpu().numpy(), g1["budget_2"]["out"], atol=2e-3 * 0.80443)
    ix.dynakv_retrieve_attend(q, 6, out, lse)
    st = ix.dynakv_export_state()
    # the same entries as the worked example; the library attends the clusters in its own order (ascending id)
    got = st["gathered"][0, :st["n_gathered"][0]].tolist()
    assert sorted(got) == sorted(g1["budget_6"]["gather"])
    order = st["selected"][0, :st["n_selected"][0]].tolist()
    assert sorted(order) == sorted(g1["budget_6"]["selected"]) if "selected" in g1["budget_6"] else len(order) == 2
    assert got == sum((g1["clusters"]["members"][j] for j in order), [])
    # example 3: append, flag, split
    cfg = binding.Config(1, 1, dtype, 2, 8, 64, kmeans_iters=3, var_alpha=1.5, buffer_max=16, softmax_scale=scale)
    ix = binding.Index(cfg, DEV)
    K = torch.from_numpy(_pad(g3["keys"]))[None].to(DEV).to(tdt)
    ix.dynakv_build_index(K, K, torch.tensor([g3["init_idx"]], dtype=torch.int32, device=DEV))
    ix.dynakv_retrieve_attend(q, 4, out, lse)
    k = torch.from_numpy(_pad([g3["new_key"]])).to(DEV).to(tdt)
    ix.dynakv_append(k, k)
    st = ix.dynakv_export_state()
    assert (st["flag"][0, 0], st["buffered"][0, 0], st["size"][0, 0], st["last_assign"][0]) == (1, 1, 4, 0)
    ix.dynakv_split()
    st = ix.dynakv_export_state()
    assert st["n_clusters"][0] == 3 and st["counters"][0, 0] == 1
    for ch in (g3["split"]["stay"], g3["split"]["moved"]):
        j = ch["id"]
        lo, hi = st["offsets"][0, j], st["offsets"][0, j + 1]
        assert st["members"][0, lo:hi].tolist() == ch["members"]
        np.testing.assert_allclose(st["centroids"][0, j, :2].numpy(), np.array(ch["centroid"], np.float32), rtol=1e-6)
        assert st["m2"][0, j] == pytest.approx(ch["M2"], abs=1e-9) and st["size"][0, j] == ch["n"]


# --------------------------------------------------------------------------- budgets, dense limit, degenerate shapes

def _dense(Q, K, V, scale):
    q, k, v = (torch.from_numpy(np.asarray(a, np.float64)) for a in (Q, K, V))
    lg = scale * torch.einsum("ugd,utd->ugt", q, k)
    return torch.einsum("ugt,utd->ugd", torch.softmax(lg, -1), v).numpy(), torch.logsumexp(lg, -1).numpy()


def _build_pair(s, w, n_units, K0=None, init=None, **over):
    ix, o = make_pair(s, n_units, **over)
    K0 = w["K0"] if K0 is None else K0
    init = w["init_idx"] if init is None else init
    ix.dynakv_build_index(to_dev(K0, s.dtype), to_dev(w["V0"], s.dtype), torch.from_numpy(init).to(DEV))
    o.build_index(K0, w["V0"], init)
    t = Tally()
    compare_build(ix, o, t, K0.shape[1])
    return ix, o, t


@pytest.mark.parametrize("dtype,G,N0,M0", [("f16", 4, 1000, 37), ("bf16", 16, 300, 300), ("f32", 1, 530, 1), ("f16", 5, 16, 16)])
def test_budget_edges_and_dense_limit(dtype, G, N0, M0):
    s = WorkloadSpec("edge", dtype, 2, G, N0, 40, M0, 10 ** 6, 8, 0.05, var_alpha=1.3, size_factor=2.0, seed=77)
    w = generate(s)
    ix, o, tally = _build_pair(s, w, 2, kmeans_iters=4)
    out = torch.empty(2, G, 128, device=DEV)
    lse = torch.empty(2, G, device=DEV)
    Qd, Kd, Vd = to_dev(w["Q"], dtype), to_dev(w["Knew"], dtype), to_dev(w["Vnew"], dtype)
    biggest = int(o.clusters(0)["n"].max())
    budgets = [0, 1, max(1, biggest - 1), biggest, N0 // 3, N0 - 1, N0 + 100, 10 ** 6]
    for t in range(s.steps):
        B = budgets[t % len(budgets)]
        ix.dynakv_retrieve_attend(Qd[t], B, out, lse)
        oo, ol = o.retrieve_attend(w["Q"][t], B)
        dirty = compare_retrieval(ix, o, tally, "edge step %d budget %d" % (t, B), Q=w["Q"][t], budget=B)
        keep = [u for u in range(2) if u not in dirty]
        check_attention(out.cpu().numpy()[keep], lse.cpu().numpy()[keep], oo[keep], ol[keep], "edge step %d budget %d" % (t, B))
        if B >= N0 + t:   # everything retrieved: dense attention over the whole cache
            allK = np.concatenate([w["K0"], w["Knew"][:t].transpose(1, 0, 2)], 1)
            allV = np.concatenate([w["V0"], w["Vnew"][:t].transpose(1, 0, 2)], 1)
            ref, rl = _dense(w["Q"][t], allK, allV, 1 / np.sqrt(128))
            check_attention(out.cpu().numpy(), lse.cpu().numpy(), ref, rl, "dense step %d" % t)
            assert not dirty
        ix.dynakv_append(Kd[t], Vd[t]); o.append(w["Knew"][t], w["Vnew"][t])
        ix.dynakv_split(); o.split()
        dirty |= compare_state(ix, o, tally, "edge step %d" % t, full=True, skip=dirty)
        parity.resync(ix, o, None, dirty, tally)
    say("edges", dtype, G, N0, M0, dict(tally))


@pytest.mark.parametrize("launch", [0, launch_shape(0, 0, LAUNCH_SEPARATE)])
def test_selection_with_equal_scores_and_large_active_sets(launch):
    """The selection's special paths: every score equal (a zero query: ids decide, and the cut falls inside the
    group of equal scores), and active sets of more than a thousand clusters."""
    s = WorkloadSpec("sel", "f16", 2, 4, 4096, 4, 1400, 10 ** 6, 8, 0.05, var_alpha=0.0, size_factor=0.0, seed=31)
    w = generate(s)
    ix, o, tally = _build_pair(s, w, 2, kmeans_iters=2, launch=launch)
    out = torch.empty(2, 4, 128, device=DEV)
    lse = torch.empty(2, 4, device=DEV)
    zero = np.zeros_like(w["Q"][0])
    cases = [("all equal", zero, B) for B in (0, 1, 7, 100, 2500, 4095, 4096, 10 ** 6)]
    cases += [("large set", w["Q"][1], B) for B in (3000, 3500, 4096, 10 ** 6)]
    cases += [("mid set", w["Q"][2], B) for B in (1, 64, 1024, 2048)]
    for what, Q, B in cases:
        ix.dynakv_retrieve_attend(to_dev(Q, "f16"), B, out, lse)
        oo, ol = o.retrieve_attend(Q, B)
        dirty = compare_retrieval(ix, o, tally, "%s budget %d" % (what, B), Q=Q, budget=B)
        assert not dirty or what != "all equal"      # exact ties go by id on both sides: never a disagreement
        keep = [u for u in range(2) if u not in dirty]
        check_attention(out.cpu().numpy()[keep], lse.cpu().numpy()[keep], oo[keep], ol[keep], "%s budget %d" % (what, B))
    st = ix.dynakv_export_state(["n_selected"])
    say("selection paths", hex(launch), "last active set:", st["n_selected"].tolist(), dict(tally))


def test_group_sum_custom_scale_all_resident_and_huge_logits():
    s = WorkloadSpec("opts", "f16", 3, 3, 700, 64, 24, 200, 6, 0.1, var_alpha=1.2, size_factor=0.0, buffer_max=0, seed=99)
    r = run_trajectory(s, range(3), 64, group_reduce=1, softmax_scale=0.05, kmeans_iters=5, full_every=8)
    say("opts:", {k: r[k] for k in ("worst_rel", "ties", "splits", "clusters")})
    assert r["splits"] > 0
    ix, o, w = r["index"], r["oracle"], r["workload"]
    Q = w["Q"][0] * 200.0                      # logits far beyond exp's range without max subtraction
    out = torch.empty(3, 3, 128, device=DEV)
    lse = torch.empty(3, 3, device=DEV)
    ix.dynakv_retrieve_attend(to_dev(Q, "f16"), 300, out, lse)
    from paper_2511_07427_amd.workload import round_to_dtype
    Qr = round_to_dtype(Q, "f16")
    oo, ol = o.retrieve_attend(Qr, 300)
    dirty = compare_retrieval(ix, o, Tally(), "huge logits", Q=Qr, budget=300)
    keep = [u for u in range(3) if u not in dirty]
    assert torch.isfinite(out).all() and torch.isfinite(lse).all()
    den = np.maximum(np.abs(oo).max(-1), 1e-6)
    assert (np.abs(out.cpu().numpy() - oo).max(-1) / den)[keep].max() <= 2e-3
    assert np.abs(lse.cpu().numpy() - ol)[keep].max() <= 2e-3 * np.abs(ol).max()


@pytest.mark.parametrize("dtype,kw", [("bf16", dict(search_copy=1)), ("f16", dict(search_copy=1, score_round=1)),
                                      ("bf16", dict(score_round=1)), ("f16", dict(update_mode=1))])
def test_readings_behind_config_fields(dtype, kw):
    """Both settings of the two readings that are configuration fields on both sides (which copy of the centroids the
    searches read, whether scores are rounded to float32 before they are compared), and the static-update mode."""
    s = CONFIGS["llama3_8b"].scaled(dtype=dtype, prefill=1536, n_clusters_init=96, budget=384, var_alpha=1.3)
    r = run_trajectory(s, [0, 1, 2], 160, check_every=2, full_every=40, step_call="mixed", kmeans_iters=4, **kw)
    say("readings", dtype, kw, {k: r[k] for k in ("worst_rel", "ties", "splits", "clusters")})
    if kw.get("update_mode"):
        assert r["splits"] == 0 and r["clusters"] == [96, 96, 96]
    else:
        assert r["splits"] > 0


@pytest.mark.parametrize("dtype,N0,M0", [("f16", 8292, 8192), ("bf16", 700, 640), ("f32", 700, 700)])
def test_token_level_mode(dtype, N0, M0):
    """The baseline without clustering: every entry its own cluster (retrieval = exact top-B over tokens), appended
    entries become new clusters; more clusters than the selection keeps in LDS, and the capacity error at the end."""
    s = CONFIGS["llama3_8b"].scaled(dtype=dtype, prefill=N0, n_clusters_init=M0, budget=300, max_cluster_factor=1)
    r = run_trajectory(s, [0, 1], 40, check_every=1, full_every=10, step_call="mixed", update_mode=2, kmeans_iters=1,
                       max_clusters=M0 + 36)
    say("token level", dtype, {k: r[k] for k in ("worst_rel", "ties", "splits", "clusters")})
    ix, o = r["index"], r["oracle"]
    st = ix.dynakv_export_state(["error", "n_clusters", "n_tokens", "size"])
    assert r["splits"] == 0 and st["n_clusters"].tolist() == [M0 + 36] * 2 and st["n_tokens"].tolist() == [N0 + 36] * 2
    assert st["error"].tolist() == [binding.ERR_CLUSTERS] * 2 and o.error(0) == 2
    assert int(st["size"][:, M0:M0 + 36].min()) == 1


@pytest.mark.parametrize("dtype,kw", [("f16", {}), ("bf16", {}), ("f32", {}), ("f16", dict(search_copy=1))])
def test_chunked_prefill_extension(dtype, kw):
    """dynakv_extend_index: k-means on the first chunk, the second chunk (drifted keys) added entry by entry with every
    cluster resident; compared with the oracle's extension, then decode steps go on from the extended index."""
    s = CONFIGS["llama3_8b"].scaled(dtype=dtype, prefill=1024, n_clusters_init=48, budget=300, var_alpha=1.25, drift_std=0.1)
    U, n2, steps = 3, 384, 24
    w = generate(s, units=range(U), steps=n2 + steps)
    ix, o = make_pair(s, U, max_tokens=1024 + n2 + steps, kmeans_iters=4, **kw)
    ix.dynakv_build_index(to_dev(w["K0"], dtype), to_dev(w["V0"], dtype), torch.from_numpy(w["init_idx"]).to(DEV))
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    tally = Tally()
    compare_build(ix, o, tally, 1024)
    K1, V1 = np.ascontiguousarray(w["Knew"][:n2].transpose(1, 0, 2)), np.ascontiguousarray(w["Vnew"][:n2].transpose(1, 0, 2))
    ix.dynakv_extend_index(to_dev(K1, dtype), to_dev(V1, dtype))
    o.extend(K1, V1)
    # the extension takes hundreds of decisions between two comparisons: a tie in any of them shows as a different
    # partition with no single margin to blame, so the comparison is strict (none occurred on these inputs)
    st = ix.dynakv_export_state(["n_clusters", "n_tokens", "flag", "members", "offsets", "error"])
    for u in range(U):
        M = o.num_clusters(u)
        off, mem = o.members(u)
        assert st["n_clusters"][u] == M > 48 and st["n_tokens"][u] == 1024 + n2 and st["error"][u] == 0
        assert int(st["flag"][u].sum()) == 0
        np.testing.assert_array_equal(st["offsets"][u, :M + 1].numpy(), off)
        np.testing.assert_array_equal(st["members"][u, :1024 + n2].numpy(), mem)
    assert not compare_state(ix, o, tally, "after the extension", assign=False)
    w2 = {k: (v[n2:] if k in ("Q", "Knew", "Vnew") else v) for k, v in w.items()}
    sp = parity.Stepper(ix, o, s, w2, None, 300)
    sp.tally = tally
    for t in range(steps):
        sp.step(t, t % 2 == 1, attention=True, full=(t % 8 == 0 or t == steps - 1))
    say("chunked prefill", dtype, kw, sp.report())


@pytest.mark.parametrize("dtype,launch", [("f16", 0), ("bf16", launch_shape(2, 0, LAUNCH_SEPARATE)), ("f32", 0)])
def test_coretrieval_placement(dtype, launch):
    """dynakv_place_by_coretrieval (Section 5.1, Eq. 8): co-retrieval probabilities and placement chain against the
    oracle's; the page pool then follows the chain, everything else (partition, statistics, retrieval results) is
    as before, and decode steps go on under the parity protocol."""
    s = CONFIGS["llama3_8b"].scaled(dtype=dtype, prefill=1536, n_clusters_init=64, budget=400, var_alpha=1.3)
    U, R, steps = 3, 24, 32
    w = generate(s, units=range(U), steps=R + steps)
    ix, o = make_pair(s, U, max_tokens=1536 + steps, kmeans_iters=4, launch=launch)
    K0, V0 = to_dev(w["K0"], dtype), to_dev(w["V0"], dtype)
    ix.dynakv_build_index(K0, V0, torch.from_numpy(w["init_idx"]).to(DEV))
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    tally = Tally()
    compare_build(ix, o, tally, 1536)
    out0, lse0 = torch.empty(U, s.group_size, 128, device=DEV), torch.empty(U, s.group_size, device=DEV)
    q_probe = to_dev(w["Q"][R], dtype)
    ix.dynakv_retrieve_attend(q_probe, 400, out0, lse0)
    before = ix.dynakv_export_state(["offsets", "members", "centroids", "m2", "size", "gathered", "n_gathered", "first_page"])
    P, order = ix.dynakv_place_by_coretrieval(K0, V0, to_dev(w["Q"][:R], dtype), 400)
    Po, oo = o.coretrieval(w["Q"][:R], 400)
    np.testing.assert_allclose(P.cpu().numpy(), Po, rtol=1e-6, atol=1e-9)
    np.testing.assert_array_equal(order.cpu().numpy(), oo)
    assert float(P.sum()) == pytest.approx(U, rel=1e-4) and int((P > 0).sum()) > 0
    out1, lse1 = torch.empty_like(out0), torch.empty_like(lse0)
    ix.dynakv_retrieve_attend(q_probe, 400, out1, lse1)
    after = ix.dynakv_export_state(["offsets", "members", "centroids", "m2", "size", "gathered", "n_gathered", "first_page", "error"])
    assert not after["error"].any()
    for k in ("offsets", "members", "centroids", "m2", "size", "gathered", "n_gathered"):
        assert torch.equal(before[k], after[k]), k
    assert torch.allclose(out0, out1, rtol=1e-6, atol=1e-7) and torch.allclose(lse0, lse1, atol=1e-6)
    fp, sz, ch = after["first_page"].numpy(), after["size"].numpy(), order.cpu().numpy()
    assert not np.array_equal(before["first_page"].numpy(), fp)
    for u in range(U):                                  # the pool follows the chain: each cluster right after its predecessor
        nxt = 0
        for j in ch[u]:
            if sz[u, j] > 0:
                assert fp[u, j] == nxt
                nxt += (sz[u, j] + 15) // 16
    o.retrieve_attend(w["Q"][R], 400)                   # the oracle's active set as the library's
    w2 = {k: (v[R:] if k in ("Q", "Knew", "Vnew") else v) for k, v in w.items()}
    sp = parity.Stepper(ix, o, s, w2, None, 400)
    sp.tally = tally
    for t in range(steps):
        sp.step(t, t % 2 == 0, attention=True, full=(t % 8 == 0 or t == steps - 1))
    say("co-retrieval placement", dtype, hex(launch), sp.report())
    # an index that has moved on since it was built is refused
    ix.dynakv_place_by_coretrieval(K0, V0, to_dev(w["Q"][:2], dtype), 400)
    st = ix.dynakv_export_state(["error"])
    assert st["error"].tolist() == [binding.ERR_PLACE] * U


@pytest.mark.parametrize("dtype,W,k", [("f16", 32, 4), ("bf16", 128, 32), ("f32", 20, 3)])
def test_local_update_mode(dtype, W, k):
    """The local-update baseline: new entries are clusters of their own until a window is full, its own k-means then
    replaces them; several windows, mixed call styles, the prefill's clusters untouched."""
    s = CONFIGS["llama3_8b"].scaled(dtype=dtype, prefill=1024, n_clusters_init=40, budget=300, max_cluster_factor=8, drift_std=0.08)
    steps = 2 * W + 9
    r = run_trajectory(s, [0, 1], steps, check_every=1, full_every=7, step_call="mixed", update_mode=3, local_window=W,
                       local_clusters=k, kmeans_iters=3)
    say("local update", dtype, W, k, {x: r[x] for x in ("worst_rel", "ties", "splits", "clusters")})
    assert r["clusters"] == [40 + 2 * k + 9] * 2 and r["splits"] == 0


def test_capacity_limits_set_the_error_word_and_keep_state():
    s = WorkloadSpec("cap", "f16", 1, 2, 64, 8, 4, 32, 4, 0.5, var_alpha=0.5, size_factor=0.0, buffer_max=0,
                     max_cluster_factor=1, seed=5)
    w = generate(s)
    ix, o, tally = _build_pair(s, w, 1, max_tokens=68)
    assert ix.export_status == binding.OK
    Kd, Vd = to_dev(w["Knew"], "f16"), to_dev(w["Vnew"], "f16")
    for t in range(8):                          # 4 appends fit, then max_tokens; splits have no free cluster id
        ix.dynakv_append(Kd[t], Vd[t]); o.append(w["Knew"][t], w["Vnew"][t])
        ix.dynakv_split(); o.split()
        assert not compare_state(ix, o, tally, "cap step %d" % t)
    st = ix.dynakv_export_state(["error", "n_tokens", "n_clusters"])
    assert ix.export_status == binding.ECAPACITY      # the sticky words leave the device as a status
    assert st["n_tokens"][0] == 68 and st["n_clusters"][0] == 4
    assert st["error"][0] & binding.ERR_TOKENS and st["error"][0] & binding.ERR_CLUSTERS
    assert "capacity" in binding.load().dynakv_strerror(binding.ECAPACITY).decode()


@pytest.mark.parametrize("launch", [0, launch_shape(0, 0, LAUNCH_SEPARATE)])
def test_whole_step_call_at_the_capacity_limits(launch):
    s = WorkloadSpec("cap", "f16", 1, 2, 64, 8, 4, 32, 4, 0.5, var_alpha=0.5, size_factor=0.0, buffer_max=0,
                     max_cluster_factor=1, seed=5)
    w = generate(s)
    ix, o, tally = _build_pair(s, w, 1, max_tokens=68, launch=launch)
    Qd, Kd, Vd = to_dev(w["Q"], "f16"), to_dev(w["Knew"], "f16"), to_dev(w["Vnew"], "f16")
    out = torch.empty(1, 2, 128, device=DEV)
    lse = torch.empty(1, 2, device=DEV)
    for t in range(8):
        ix.dynakv_decode_step(Qd[t], 32, out, lse, Kd[t], Vd[t])
        oo, ol = o.retrieve_attend(w["Q"][t], 32)
        assert not compare_retrieval(ix, o, tally, "cap step %d" % t, gather=False, Q=w["Q"][t], budget=32)
        check_attention(out.cpu().numpy(), lse.cpu().numpy(), oo, ol, "cap step %d" % t)
        o.append(w["Knew"][t], w["Vnew"][t]); o.split()
        assert not compare_state(ix, o, tally, "cap step %d" % t)
    st = ix.dynakv_export_state(["error", "n_tokens"])
    assert st["n_tokens"][0] == 68 and st["error"][0] & binding.ERR_TOKENS and ix.export_status == binding.ECAPACITY


def test_initial_positions_out_of_range_or_repeated_set_the_error_word():
    s = CONFIGS["tiny"].scaled(prefill=300, n_clusters_init=12)
    w = generate(s, steps=1)
    ix, _ = make_pair(s, 1)
    K0, V0 = to_dev(w["K0"], "f32"), to_dev(w["V0"], "f32")
    for bad, want in ((None, 0), ((3, 300), binding.ERR_INIT), ((5, -1), binding.ERR_INIT), ((7, "dup"), binding.ERR_INIT)):
        init = w["init_idx"].copy()
        if bad:
            init[0, bad[0]] = init[0, 0] if bad[1] == "dup" else bad[1]
        ix.dynakv_build_index(K0, V0, torch.from_numpy(init).to(DEV))
        st = ix.dynakv_export_state(["error", "n_clusters", "n_tokens"])
        assert st["error"][0] == want and st["n_clusters"][0] == 12 and st["n_tokens"][0] == 300, bad
        assert ix.export_status == (binding.ECAPACITY if want else binding.OK)


def test_prefill_with_a_wide_key_range():
    """Keys whose exponents span far more bits than a float64 sum keeps exact (bfloat16, a few keys scaled far up
    and far down): the centres are still float64 sums of the members."""
    s = WorkloadSpec("wide", "bf16", 2, 2, 1500, 4, 24, 256, 6, 0.05, var_alpha=0.0, size_factor=0.0, seed=123)
    w = generate(s)
    K0 = w["K0"].copy()
    K0[:, 5] *= 2.0 ** 30
    K0[:, 77] *= 2.0 ** 30
    K0[:, 300:303] *= 2.0 ** -40
    ix, o, tally = _build_pair(s, w, 2, K0=K0, kmeans_iters=5)
    say("wide range", dict(tally))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_prefill_with_coinciding_centres(dtype):
    """Keys drawn from a handful of distinct vectors, so that many initial centres coincide: points whose nearest
    centre is one of several equal ones (lowest id wins on both sides: exact ties are not disagreements)."""
    s = WorkloadSpec("dup", dtype, 2, 2, 900, 4, 40, 256, 6, 0.05, var_alpha=0.0, size_factor=0.0, seed=321)
    w = generate(s)
    K0 = w["K0"].copy()
    for u, distinct in enumerate((3, 11)):
        base = K0[u, :distinct].copy()
        K0[u, :600] = base[np.arange(600) % distinct]          # the remaining 300 keys stay as drawn
    init = np.tile(np.arange(40, dtype=np.int32), (2, 1))      # the first 40 keys: 3 resp. 11 distinct centres
    ix, o, tally = _build_pair(s, w, 2, K0=K0, init=init, kmeans_iters=4)
    assert tally["tie_kmeans"] == 0


def test_rebuild_resets_the_index_and_runs_are_deterministic():
    s = CONFIGS["tiny"].scaled(prefill=777, n_clusters_init=19)
    w = generate(s, steps=8)
    ix, o = make_pair(s, 1)
    K0, V0, init = to_dev(w["K0"], "f32"), to_dev(w["V0"], "f32"), torch.from_numpy(w["init_idx"]).to(DEV)
    ix.dynakv_build_index(K0, V0, init)
    for t in range(8):
        ix.dynakv_append(to_dev(w["Knew"][t], "f32"), to_dev(w["Vnew"][t], "f32"))
    a = ix.dynakv_export_state()
    ix.dynakv_build_index(K0, V0, init)
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    compare_build(ix, o, Tally(), 777)
    for t in range(8):
        ix.dynakv_append(to_dev(w["Knew"][t], "f32"), to_dev(w["Vnew"][t], "f32"))
    b = ix.dynakv_export_state()
    for k in a:
        assert torch.equal(a[k], b[k]), k


def test_timing_aid_brackets_an_even_sample_of_the_launches():
    s = CONFIGS["llama3_8b"].scaled(prefill=512, n_clusters_init=32, budget=128)
    U = 2
    w = generate(s, units=range(U), steps=32)
    ix = binding.Index(binding.Config(U, s.group_size, s.dtype, 32, 128, 512 + 32, 3, 16, 0, s.var_alpha, s.size_factor, 0.0), DEV)
    ix.dynakv_build_index(to_dev(w["K0"], s.dtype), to_dev(w["V0"], s.dtype), torch.from_numpy(w["init_idx"]).to(DEV))
    Qd, Kd, Vd = to_dev(w["Q"], s.dtype), to_dev(w["Knew"], s.dtype), to_dev(w["Vnew"], s.dtype)
    out, lse = torch.empty(U, s.group_size, 128, device=DEV), torch.empty(U, s.group_size, device=DEV)
    lib = binding.load()
    assert lib.dynakv_profile_sample(ix._h, 0, 1) == binding.EINVAL and lib.dynakv_profile_sample(ix._h, 4, 5) == binding.EINVAL
    t = 0
    for every, run, steps, want in ((1, 1, 6, 6), (4, 2, 10, 6), (4, 4, 7, 4), (3, 1, 6, 2)):
        ix.dynakv_profile_sample(every, run)
        ix.dynakv_profile_enable(16)
        for _ in range(steps):
            ix.dynakv_decode_step(Qd[t], 128, out, lse, Kd[t], Vd[t])
            t += 1
        n, ms = ix.dynakv_profile_read()
        assert n == want and 0.0 < ms < 50.0, (every, run, steps, n, ms)
    ix.dynakv_profile_sample(1, 1)
    ix.dynakv_profile_enable(0)


# --------------------------------------------------------------------------- exported and imported state

@pytest.mark.parametrize("name,launch", [("llama3_8b", 0), ("tiny", 0), ("qwen25_7b", launch_shape(2, 0, LAUNCH_SEPARATE))])
def test_imported_state_continues_like_the_exporting_index(name, launch):
    """dynakv_export_state -> dynakv_import_state into a second index: both then take the same steps and must
    agree on every decision and, since both run the same kernels on the same values, on every exported bit
    except the page-dependent gather order inside a step."""
    s = CONFIGS[name].scaled(prefill=1024, n_clusters_init=48, budget=256, var_alpha=1.25 if name != "tiny" else 0.0)
    U = 3
    w = generate(s, units=range(U), steps=96)
    mk = lambda: binding.Index(binding.Config(U, s.group_size, s.dtype, 48, 192, 1024 + 96, 4, 4, 0, s.var_alpha,
                                              s.size_factor, 0.0, launch=launch), DEV)
    a, b = mk(), mk()
    a.dynakv_build_index(to_dev(w["K0"], s.dtype), to_dev(w["V0"], s.dtype), torch.from_numpy(w["init_idx"]).to(DEV))
    Qd, Kd, Vd = to_dev(w["Q"], s.dtype), to_dev(w["Knew"], s.dtype), to_dev(w["Vnew"], s.dtype)
    oa, la = torch.empty(U, s.group_size, 128, device=DEV), torch.empty(U, s.group_size, device=DEV)
    ob, lb = torch.empty_like(oa), torch.empty_like(la)
    for t in range(48):
        a.dynakv_decode_step(Qd[t], 256, oa, la, Kd[t], Vd[t])
    a.dynakv_retrieve_attend(Qd[48], 256, oa, la)              # the active set travels with the state
    snap = a.dynakv_export_state(binding.IMPORT_FIELDS, to_cpu=False)
    if name == "llama3_8b":
        assert int(snap["flag"].sum()) > 0                     # flagged clusters and their buffers are part of it
    b.dynakv_import_state(snap)
    fields = ("n_clusters", "n_tokens", "error", "tau", "centroids", "size", "buffered", "flag", "m2", "offsets", "members",
              "keys", "values")
    sa, sb = a.dynakv_export_state(fields), b.dynakv_export_state(fields)
    for k in fields:
        assert torch.equal(sa[k], sb[k]), "right after the import: " + k
    for ix in (a, b):
        ix.dynakv_append(Kd[48], Vd[48]); ix.dynakv_split()
    for t in range(49, 96):
        a.dynakv_decode_step(Qd[t], 256, oa, la, Kd[t], Vd[t])
        b.dynakv_decode_step(Qd[t], 256, ob, lb, Kd[t], Vd[t])
        assert torch.allclose(oa, ob, rtol=2e-3, atol=1e-6) and torch.allclose(la, lb, atol=2e-3), t
    sa, sb = a.dynakv_export_state(fields + ("scores", "n_selected", "n_gathered")), b.dynakv_export_state(fields + ("scores", "n_selected", "n_gathered"))
    for k in sa:
        assert torch.equal(sa[k], sb[k]), k
    assert int(sa["n_clusters"].max()) > 48
    # an inconsistent snapshot is refused unit by unit and leaves the index as it was
    snap["n_clusters"][1] = 10 ** 6
    snap["offsets"][2, 1] += 1
    b.dynakv_import_state(snap)
    sb2 = b.dynakv_export_state(("error", "n_clusters", "n_tokens", "members"))
    assert b.export_status == binding.ECAPACITY
    assert sb2["error"].tolist() == [0, binding.ERR_IMPORT, binding.ERR_IMPORT]
    assert torch.equal(sb2["members"][1:], sb["members"][1:]) and torch.equal(sb2["n_tokens"][1:], sb["n_tokens"][1:])
    assert int(sb2["n_tokens"][0]) == 1024 + 48
