"""Pins of the CPU oracle against things other than itself (CPU only).

Library routines on special cases (scipy cdist, scikit-learn Lloyd, torch dense attention), closed forms,
invariants of the partition (Eq. 3), brute force on tiny inputs and hand-computed fixtures.
"""
import json
import os

import numpy as np
import pytest
import torch
from scipy.spatial.distance import cdist

from oracle import Oracle, OracleConfig
from paper_2511_07427_amd.workload import CONFIGS, generate

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def cfg(U=1, G=1, d=2, M0=2, maxc=8, maxt=64, iters=3, bmax=16, alpha=0.0, size=0.0, reduce=0, scale=0.0, **kw):
    return OracleConfig(U, G, d, M0, maxc, maxt, iters, bmax, reduce, alpha, size, scale, **kw)


def blobs(rng, n, d, k, sep=6.0, std=0.5):
    c = rng.standard_normal((k, d)) * sep
    lab = rng.integers(0, k, n)
    return (c[lab] + std * rng.standard_normal((n, d))).astype(np.float32), c


def dense_attention(Q, K, V, scale):
    q, k, v = (torch.from_numpy(np.asarray(a, np.float64)) for a in (Q, K, V))
    out = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], scale=scale)[0]
    lse = torch.logsumexp(scale * q @ k.T, dim=-1)
    return out.numpy(), lse.numpy()


# ---------------------------------------------------------------- k-means (Section 4.1, Eq. 3-4)

def test_assignment_is_cdist_argmin():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((1, 500, 16)).astype(np.float32)
    init = rng.choice(500, 24, replace=False)[None].astype(np.int32)
    o = Oracle(cfg(d=16, M0=24, maxc=24, maxt=500, iters=1))
    J = o.build_index(X, X, init)
    D = cdist(X[0].astype(np.float64), X[0][init[0]].astype(np.float64), "sqeuclidean")
    np.testing.assert_array_equal(o.labels(0), D.argmin(1))
    assert J[0, 0] == pytest.approx(D.min(1).sum(), rel=1e-12)


def test_lloyd_matches_sklearn_and_objective_decreases():
    from sklearn.cluster import KMeans
    rng = np.random.default_rng(2)
    X, _ = blobs(rng, 600, 8, 6)
    init = rng.choice(600, 6, replace=False).astype(np.int32)
    T = 5
    o = Oracle(cfg(d=8, M0=6, maxc=6, maxt=600, iters=T))
    J = o.build_index(X[None], X[None], init[None])
    assert np.all(np.diff(J[0]) <= 1e-9 * J[0, 0])
    Xd = X.astype(np.float64)
    full = KMeans(6, init=Xd[init], n_init=1, algorithm="lloyd", max_iter=T, tol=0).fit(Xd)
    prev = KMeans(6, init=Xd[init], n_init=1, algorithm="lloyd", max_iter=T - 1, tol=0).fit(Xd)
    c = o.clusters(0)
    assert c["n"].min() > 0
    # centres after T updates; labels are those of the T-th assignment (= against the centres after T-1 updates)
    np.testing.assert_allclose(c["centroids"], full.cluster_centers_, rtol=1e-6, atol=1e-6)
    np.testing.assert_array_equal(o.labels(0), prev.labels_)


def test_kmeans_closed_forms():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((1, 200, 5)).astype(np.float32)
    o = Oracle(cfg(d=5, M0=1, maxc=2, maxt=200, iters=2))
    J = o.build_index(X, X, np.zeros((1, 1), np.int32))
    Xd = X[0].astype(np.float64)
    np.testing.assert_allclose(o.clusters(0)["centroids"][0], Xd.mean(0), rtol=1e-6, atol=1e-7)
    assert J[0, 1] == pytest.approx(200 * np.trace(np.cov(Xd.T, bias=True)), rel=1e-6)
    assert o.clusters(0)["M2"][0] == pytest.approx(J[0, 1], rel=1e-6)
    # every point its own centre: objective 0, each cluster one member
    o = Oracle(cfg(d=5, M0=200, maxc=200, maxt=200, iters=2))
    J = o.build_index(X, X, np.arange(200, dtype=np.int32)[None])
    assert J[0, 0] == 0.0 and J[0, 1] == 0.0
    np.testing.assert_array_equal(o.labels(0), np.arange(200))


def test_centroid_is_member_mean_and_variance_is_mean_sqdist():
    s = CONFIGS["tiny"]
    w = generate(s)
    o = Oracle(OracleConfig(1, 4, 128, 32, 128, s.max_tokens, 10, 16, 0, 1.5, 0.0, 0.0))
    J = o.build_index(w["K0"], w["V0"], w["init_idx"])
    assert np.all(np.diff(J[0]) <= 0)
    c, (off, mem) = o.clusters(0), o.members(0)
    X = w["K0"][0].astype(np.float64)
    tot = 0.0
    for j in range(32):
        m = mem[off[j]:off[j + 1]]
        assert len(m) == c["n"][j] and np.all(np.diff(m) > 0)
        np.testing.assert_allclose(c["centroids"][j], X[m].mean(0), rtol=2e-7, atol=1e-7)       # Eq. 4
        ss = ((X[m] - c["centroids"][j].astype(np.float64)) ** 2).sum()
        assert c["M2"][j] == pytest.approx(ss, rel=1e-12)
        tot += ss
    assert o.tau(0) == pytest.approx(1.5 * tot / 2048, rel=1e-12)
    assert sorted(mem.tolist()) == list(range(2048))                                          # Eq. 3


def test_empty_cluster_is_reseeded_with_the_farthest_point():
    # two coincident initial centres: the second gets no point in iteration 1 and must take the farthest one
    X = np.array([[0, 0], [0, 0], [1, 0], [0, 1], [50, 50]], np.float32)[None]
    o = Oracle(cfg(M0=2, iters=3, maxt=5))
    J = o.build_index(X, X, np.array([[0, 1]], np.int32))
    assert np.all(np.diff(J[0]) <= 0)
    np.testing.assert_array_equal(o.labels(0), [0, 0, 0, 0, 1])
    np.testing.assert_allclose(o.clusters(0)["centroids"], [[0.25, 0.25], [50, 50]])


# ---------------------------------------------------------------- hand examples

def _example1():
    g = json.load(open(os.path.join(GOLD, "hand_example_1_retrieve.json")))
    K = np.array(g["keys"], np.float32)[None]
    V = np.array(g["values"], np.float32)[None]
    return g, K, V


def test_hand_example_1_build_select_attend():
    g, K, V = _example1()
    o = Oracle(cfg(maxt=16))
    o.build_index(K, V, np.array([g["init_idx"]], np.int32))
    c, (off, mem) = o.clusters(0), o.members(0)
    for j, m in enumerate(g["clusters"]["members"]):
        assert mem[off[j]:off[j + 1]].tolist() == m
    np.testing.assert_allclose(c["centroids"], g["clusters"]["centroids"], rtol=0, atol=0)
    assert c["n"].tolist() == g["clusters"]["n"]
    np.testing.assert_allclose(c["M2"], g["clusters"]["M2"], rtol=1e-15)
    np.testing.assert_allclose(c["M2"] / c["n"], g["clusters"]["variance"], rtol=1e-15)
    q = np.array(g["query"], np.float32)[None, None]
    out, lse = o.retrieve_attend(q, 2)
    np.testing.assert_allclose(o.scores(0), g["scores"], rtol=1e-7)
    assert o.selected(0).tolist() == g["budget_2"]["selected"]
    assert o.gather(0).tolist() == g["budget_2"]["gather"]
    np.testing.assert_allclose(out[0, 0], g["budget_2"]["out"], atol=1e-7)
    out, lse = o.retrieve_attend(q, 6)
    assert o.selected(0).tolist() == g["budget_6"]["selected"]
    assert o.gather(0).tolist() == g["budget_6"]["gather"]
    ref, rl = dense_attention(q[0], K[0], V[0], 1 / np.sqrt(2))
    np.testing.assert_allclose(out[0], ref, rtol=1e-12)
    np.testing.assert_allclose(lse[0], rl, rtol=1e-12)
    # budget between the two sizes: the better cluster fits, the next does not, nothing is skipped or cut
    out, _ = o.retrieve_attend(q, 5)
    assert o.selected(0).tolist() == [1]


def test_hand_example_2_updatevar_and_flag():
    g1, K, V = _example1()
    g = json.load(open(os.path.join(GOLD, "hand_example_2_updatevar.json")))
    k = np.array([g["new_key"]], np.float32)
    D = cdist(k.astype(np.float64), np.array(g1["clusters"]["centroids"]), "sqeuclidean")[0]
    np.testing.assert_allclose(D, g["sqdist_to_centroids"])
    pts = np.array(g1["keys"][:4] + [g["new_key"]], np.float64)
    np.testing.assert_allclose(((pts - g["tentative"]["centroid"]) ** 2).sum(1), g["tentative"]["two_pass_sqdist"])
    assert sum(g["tentative"]["two_pass_sqdist"]) == pytest.approx(g["tentative"]["M2"])

    o = Oracle(cfg(maxt=16, alpha=g["var_alpha"]))
    o.build_index(K, V, np.array([g1["init_idx"]], np.int32))
    assert o.tau(0) == pytest.approx(g["tau"], rel=1e-15)
    o.retrieve_attend(np.array([[[-1, -1]]], np.float32), 1)   # active set without cluster 0
    o.append(k, k)
    assert o.last_assign(0) == g["assigned"]
    c, (off, mem) = o.clusters(0), o.members(0)
    a = g["after"]
    assert (c["flag"][0], c["b"][0], c["n"][0]) == (a["flag"], a["b"], a["n"])
    np.testing.assert_array_equal(c["centroids"][0], np.array(a["centroid"], np.float32))
    assert c["M2"][0] == a["M2"]
    assert mem[off[0]:off[1]].tolist() == a["members"]
    assert o.diagnostics(0)["margin_trigger"] == pytest.approx((0.8 - 0.75) / 1.0)
    # a second entry of a flagged cluster only grows the buffer
    o.append(np.array([[0.5, 0.5]], np.float32), k)
    c = o.clusters(0)
    assert (c["flag"][0], c["b"][0], c["n"][0]) == (1, 2, 4)

    b = g["with_tau_above"]
    o = Oracle(cfg(maxt=16, alpha=b["var_alpha"]))
    o.build_index(K, V, np.array([g1["init_idx"]], np.int32))
    o.append(k, k)
    c = o.clusters(0)
    assert (c["flag"][0], c["b"][0], c["n"][0]) == (b["flag"], b["b"], b["n"])
    np.testing.assert_allclose(c["centroids"][0], b["centroid"], rtol=1e-7)
    assert c["M2"][0] == pytest.approx(b["M2"], rel=1e-7)


@pytest.mark.parametrize("bmax", [0, 16])
def test_hand_example_3_split(bmax):
    g = json.load(open(os.path.join(GOLD, "hand_example_3_split.json")))
    K = np.array(g["keys"], np.float32)[None]
    o = Oracle(cfg(maxt=16, alpha=1.5, bmax=bmax))
    o.build_index(K, K, np.array([g["init_idx"]], np.int32))
    k = np.array([g["new_key"]], np.float32)
    o.retrieve_attend(np.array([[[1, 1]]], np.float32), 4)    # active set = {cluster 0}
    assert o.selected(0).tolist() == [0]
    o.append(k, k)
    assert o.last_assign(0) == g["assigned"]
    c = o.clusters(0)
    assert (c["flag"][0], c["b"][0], c["n"][0]) == (1, 1, 4)
    o.split()
    assert o.num_clusters(0) == 3
    c, (off, mem) = o.clusters(0), o.members(0)
    for ch in (g["split"]["stay"], g["split"]["moved"]):
        j = ch["id"]
        assert mem[off[j]:off[j + 1]].tolist() == ch["members"]
        np.testing.assert_array_equal(c["centroids"][j], np.array(ch["centroid"], np.float32))
        assert (c["n"][j], c["b"][j], c["flag"][j]) == (ch["n"], 0, 0)
        assert c["M2"][j] == pytest.approx(ch["M2"], abs=1e-15)
    assert o.diagnostics(0)["splits"] == 1


def test_delayed_split_waits_for_retrieval_and_forced_split_fires_at_bmax():
    g = json.load(open(os.path.join(GOLD, "hand_example_3_split.json")))
    K = np.array(g["keys"], np.float32)[None]
    o = Oracle(cfg(maxt=32, alpha=1.5, bmax=3))
    o.build_index(K, K, np.array([g["init_idx"]], np.int32))
    far = np.array([[[-10, -11]]], np.float32)                 # retrieves cluster 1 only (budget 2)
    k = np.array([g["new_key"]], np.float32)
    for step in range(3):
        o.retrieve_attend(far, 2)
        assert o.selected(0).tolist() == [1]
        o.append(k + step, k)
        o.split()
        c = o.clusters(0)
        if step < 2:                                          # buffered, not split: cluster 0 is not resident
            assert (c["flag"][0], c["b"][0], o.num_clusters(0)) == (1, step + 1, 2)
            assert c["n"][0] == 4 and c["M2"][0] == 2.0
    d = o.diagnostics(0)
    assert (d["splits"], d["forced_splits"], o.num_clusters(0)) == (1, 1, 3)
    off, mem = o.members(0)
    assert mem[off[0]:off[1]].tolist() == [0, 1, 2, 3] and mem[off[2]:off[3]].tolist() == [6, 7, 8]
    c = o.clusters(0)
    assert c["flag"].sum() == 0 and c["b"].sum() == 0
    # same inputs, but the flagged cluster is retrieved at step 2: the delayed split happens there
    o = Oracle(cfg(maxt=32, alpha=1.5, bmax=16))
    o.build_index(K, K, np.array([g["init_idx"]], np.int32))
    o.retrieve_attend(far, 2); o.append(k, k); o.split()
    assert o.num_clusters(0) == 2
    o.retrieve_attend(np.array([[[1, 1]]], np.float32), 5); o.append(k + 1, k); o.split()
    assert o.num_clusters(0) == 3 and o.diagnostics(0)["forced_splits"] == 0
    off, mem = o.members(0)
    assert mem[off[2]:off[3]].tolist() == [6, 7]


def test_ties_go_to_the_lowest_index():
    K = np.array([[0, 0], [2, 0], [0, 0.5], [2, 0.5]], np.float32)[None]
    o = Oracle(cfg(M0=2, iters=1, maxt=8))
    o.build_index(K, K, np.array([[0, 1]], np.int32))
    np.testing.assert_allclose(o.clusters(0)["centroids"], [[0, 0.25], [2, 0.25]])
    o.append(np.array([[1, 0.25]], np.float32), np.zeros((1, 2), np.float32))    # equidistant
    assert o.last_assign(0) == 0
    out, _ = o.retrieve_attend(np.array([[[0, 1]]], np.float32), 2)              # equal scores, budget for one
    assert o.selected(0).tolist() == [0]


# ---------------------------------------------------------------- triggers, unsplittable clusters, forced-split ties

def test_hand_example_4_size_trigger_at_its_exact_boundary():
    g = json.load(open(os.path.join(GOLD, "hand_example_4_size_trigger.json")))
    K = np.array(g["keys"], np.float32)[None]
    o = Oracle(cfg(M0=4, maxt=16, size=g["size_factor"], bmax=16))
    o.build_index(K, K, np.array([g["init_idx"]], np.int32))
    off, mem = o.members(0)
    assert [mem[off[j]:off[j + 1]].tolist() for j in range(4)] == g["clusters"]["members"]
    for step in (g["step_a"], g["step_b"]):
        assert step["lhs_n_prime_times_M"] == step["n_prime"] * step["M"]
        assert step["rhs_factor_times_N_plus_1"] == g["size_factor"] * step["N_plus_1"]
        assert o.num_tokens(0) + 1 == step["N_plus_1"] and o.num_clusters(0) == step["M"]
        k = np.array([step["new_key"]], np.float32)
        o.append(k, k)
        c = o.clusters(0)
        assert o.last_assign(0) == step["assigned"]
        assert (c["flag"][0], c["n"][0], c["b"][0]) == (step["flag"], step["n_after"], step["b_after"]), step


def _import_fixture(o, keys, clusters, selected=(), tau=0.0):
    keys = np.array(keys, np.float32)
    mem = sum((c["members"] for c in clusters), [])
    off = np.cumsum([0] + [len(c["members"]) for c in clusters])
    o.import_unit(0, keys, keys, np.array([c["centroid"] for c in clusters], np.float32), [c["n"] for c in clusters],
                  [c["b"] for c in clusters], [c["flag"] for c in clusters], [c["M2"] for c in clusters], off, mem, tau,
                  selected)


def test_hand_example_5_forced_split_tie_goes_to_the_lowest_id():
    g = json.load(open(os.path.join(GOLD, "hand_example_5_forced_tie_and_unsplittable.json")))["forced_tie"]
    o = Oracle(cfg(maxt=16, alpha=1.5, bmax=g["buffer_max"]))
    _import_fixture(o, g["keys"], g["clusters"], g["selected"], tau=1.0)
    o.split()
    a = g["after"]
    d = o.diagnostics(0)
    assert (o.num_clusters(0), d["forced_splits"], d["splits"], d["failed_splits"]) == (a["n_clusters"], 1, 1, 0)
    c, (off, mem) = o.clusters(0), o.members(0)
    for j, key in ((0, "cluster_0"), (1, "cluster_1"), (3, "cluster_3")):
        w = a[key]
        assert mem[off[j]:off[j + 1]].tolist() == w["members"]
        assert (c["n"][j], c["flag"][j], c["b"][j]) == (w["n"], w["flag"], w["b"])
        if "centroid" in w:
            np.testing.assert_array_equal(c["centroids"][j], np.array(w["centroid"], np.float32))
            assert c["M2"][j] == pytest.approx(w["M2"], abs=1e-15)


def test_hand_example_5_unsplittable_clusters_are_unflagged_with_exact_statistics():
    g = json.load(open(os.path.join(GOLD, "hand_example_5_forced_tie_and_unsplittable.json")))
    # all members equal: flagged by the size trigger, 2-means finds no second seed
    e = g["all_equal"]
    K = np.array(e["keys"], np.float32)[None]
    o = Oracle(cfg(maxt=16, size=e["size_factor"], bmax=0))
    o.build_index(K, K, np.array([e["init_idx"]], np.int32))
    k = np.array([e["new_key"]], np.float32)
    o.append(k, k)
    c = o.clusters(0)
    assert (c["flag"][0], c["b"][0], c["n"][0]) == tuple(e["after_append"][x] for x in ("flag", "b", "n"))
    o.split()
    a, c, d = e["after_split"], o.clusters(0), o.diagnostics(0)
    assert (o.num_clusters(0), d["failed_splits"], d["splits"]) == (a["n_clusters"], a["failed_splits"], a["splits"])
    assert (c["flag"][0], c["b"][0], c["n"][0], c["M2"][0]) == (a["flag"], a["b"], a["n"], a["M2"])
    np.testing.assert_array_equal(c["centroids"][0], np.array(a["centroid"], np.float32))
    assert o.members(0)[1][:6].tolist() == [0, 1, 2, 3, 4, 6]
    # a flagged cluster with a single entry (only reachable through an imported state)
    e = g["single_member"]
    o = Oracle(cfg(maxt=16, alpha=1.5, bmax=0))
    _import_fixture(o, e["keys"], e["clusters"], tau=1.0)
    o.split()
    a, c, d = e["after_split"], o.clusters(0), o.diagnostics(0)
    assert (o.num_clusters(0), d["failed_splits"], d["splits"]) == (a["n_clusters"], a["failed_splits"], 0)
    assert (c["flag"][0], c["b"][0], c["n"][0], c["M2"][0]) == (a["flag"], a["b"], a["n"], a["M2"])
    np.testing.assert_array_equal(c["centroids"][0], np.array(a["centroid"], np.float32))


def test_two_means_of_a_split_is_sklearn_lloyd_from_the_same_seeds():
    """A 2-means that needs several Lloyd rounds: partition and centres against scikit-learn started from the two
    seeds (member farthest from the mean, member farthest from that one)."""
    from sklearn.cluster import KMeans
    rounds_seen = []
    for seed in range(12):
        rng = np.random.default_rng(100 + seed)
        m, d = 90, 6
        X = np.concatenate([rng.standard_normal((m // 2, d)) * [4, 1, 1, 1, 1, 1],
                            rng.standard_normal((m - m // 2, d)) * [1, 4, 1, 1, 1, 1] + [2.5, 2.5, 0, 0, 0, 0]])
        X = X[rng.permutation(m)].astype(np.float32)
        o = Oracle(cfg(d=d, M0=1, maxc=4, maxt=m + 1, iters=1, size=0.5, bmax=0))
        o.build_index(X[None, :m - 1], X[None, :m - 1], np.zeros((1, 1), np.int32))
        o.append(X[None, m - 1], X[None, m - 1])
        assert o.clusters(0)["flag"][0] == 1
        o.split()
        assert o.num_clusters(0) == 2 and o.diagnostics(0)["splits"] == 1
        rounds_seen.append(o.last_split_rounds(0))
        Xd = X.astype(np.float64)
        a = int(((Xd - Xd.mean(0)) ** 2).sum(1).argmax())
        b = int(((Xd - Xd[a]) ** 2).sum(1).argmax())
        km = KMeans(2, init=Xd[[a, b]], n_init=1, algorithm="lloyd", max_iter=16, tol=0).fit(Xd)
        assert km.n_iter_ < 16
        lab = o.labels(0)
        same = lab == lab[0]
        np.testing.assert_array_equal(same, km.labels_ == km.labels_[0])
        c = o.clusters(0)
        for j in (0, 1):
            np.testing.assert_allclose(c["centroids"][j], Xd[lab == j].mean(0), rtol=1e-6, atol=1e-6)
        np.testing.assert_allclose(sorted(c["M2"]), sorted(((Xd[km.labels_ == s] - km.cluster_centers_[s]) ** 2).sum()
                                                          for s in (0, 1)), rtol=1e-9)
    assert max(rounds_seen) >= 4 and sum(r >= 3 for r in rounds_seen) >= 4, rounds_seen


def test_reported_margins_on_the_hand_examples():
    """The normalised margins that classify a disagreement as a tie: gap / max(1, |taken|, |runner-up|) on
    z = 2 k.r - |r|^2 for nearest-cluster decisions, on the scores around the budget cut, |variance - tau| /
    max(1, tau) for the threshold, and for a split the smallest over its seed choices and side decisions."""
    g1, K, V = _example1()
    o = Oracle(cfg(maxt=16))
    o.build_index(K, V, np.array([g1["init_idx"]], np.int32))
    o.retrieve_attend(np.array(g1["query"], np.float32)[None, None], 2)
    assert o.diagnostics(0)["margin_select"] == pytest.approx(20.0 / 21.0, rel=1e-12)    # scores 21/sqrt2 and 1/sqrt2
    k = np.array([[1, 2]], np.float32)
    o.append(k, k)
    # squared distances 2.5 and 162, |k|^2 = 5: z = 2.5 and -157
    assert o.diagnostics(0)["margin_assign"] == pytest.approx(159.5 / 157.0, rel=1e-12)
    g3 = json.load(open(os.path.join(GOLD, "hand_example_3_split.json")))
    K3 = np.array(g3["keys"], np.float32)[None]
    o = Oracle(cfg(maxt=16, alpha=1.5, bmax=0))
    o.build_index(K3, K3, np.array([g3["init_idx"]], np.int32))
    k = np.array([g3["new_key"]], np.float32)
    o.append(k, k)
    o.split()
    # seed B: distances to (9,9) are 162, 145, 145, 128, 0: gap 17 over 162 is the smallest margin of this split
    assert o.diagnostics(0)["margin_split"] == pytest.approx(17.0 / 162.0, rel=1e-12)
    assert o.last_split_rounds(0) == 1


def test_static_update_never_flags_and_config_fields_select_the_readings():
    s = CONFIGS["tiny"].scaled(dtype="bf16", var_alpha=1.2, size_factor=2.0)
    w = generate(s, steps=64)
    base = dict(n_units=1, group_size=4, head_dim=128, n_clusters_init=32, max_clusters=128, max_tokens=s.prefill + 64,
                kmeans_iters=3, buffer_max=4, var_alpha=1.2, size_factor=2.0, dtype="bf16")
    runs = {}
    for name, kw in (("copy", {}), ("mean", dict(search_copy=1)), ("round", dict(score_round=1)),
                     ("static", dict(update_mode=1))):
        o = Oracle(OracleConfig(**base, **kw))
        o.build_index(w["K0"], w["V0"], w["init_idx"])
        for t in range(64):
            o.retrieve_attend(w["Q"][t], 256)
            if t == 0:
                q = w["Q"][0, 0].astype(np.float64)
                r = (o.search_copy(0) if name != "mean" else o.clusters(0)["centroids"]).astype(np.float64)
                want = (q @ r.T).max(0) / np.sqrt(128)
                if name == "round":
                    np.testing.assert_array_equal(o.scores(0), want.astype(np.float32).astype(np.float64))
                else:
                    np.testing.assert_allclose(o.scores(0), want, rtol=1e-13)
            o.append(w["Knew"][t], w["Vnew"][t])
            o.split()
        runs[name] = o
    np.testing.assert_array_equal(runs["mean"].search_copy(0), runs["mean"].clusters(0)["centroids"])
    assert not np.array_equal(runs["copy"].search_copy(0), runs["copy"].clusters(0)["centroids"])
    st = runs["static"]
    assert st.num_clusters(0) == 32 and st.clusters(0)["flag"].sum() == 0 and st.clusters(0)["n"].sum() == s.prefill + 64
    assert runs["copy"].num_clusters(0) > 32


def test_token_level_mode_retrieves_the_exact_top_b_tokens():
    """update_mode = 2 (no clustering): every entry is its own cluster, so the selected entries are the B entries
    with the largest scores max_g <q_g, k> (brute force over all tokens), appended ones included."""
    s = CONFIGS["tiny"].scaled(prefill=300, n_clusters_init=300)
    w = generate(s, steps=40)
    o = Oracle(OracleConfig(1, 4, 128, 300, 400, 340, 1, 16, 0, 1.5, 2.0, 0.0, search_copy=1, update_mode=2))
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    assert o.clusters(0)["n"].tolist() == [1] * 300
    for t in range(40):
        o.retrieve_attend(w["Q"][t], 37)
        allK = np.concatenate([w["K0"][0], w["Knew"][:t, 0]]).astype(np.float64)
        sc = (w["Q"][t, 0].astype(np.float64) @ allK.T).max(0)
        want = np.argsort(-sc, kind="stable")[:37]
        assert sorted(o.gather(0).tolist()) == sorted(want.tolist())
        o.append(w["Knew"][t], w["Vnew"][t])
        o.split()
        assert o.num_clusters(0) == 301 + t and o.last_assign(0) == 300 + t
    c = o.clusters(0)
    assert c["flag"].sum() == 0 and c["M2"].sum() == 0.0 and c["n"].sum() == 340
    np.testing.assert_array_equal(c["centroids"][300:], w["Knew"][:, 0])


def test_chunked_prefill_extension_keeps_the_partition_and_splits_at_once():
    """Adaptive clustering through a long prefill: the first chunk is clustered by k-means, the rest is added entry by
    entry with every cluster resident.  Invariants (every token in exactly one cluster, no flag left, Eq. 4 and the
    two-pass variance on every cluster that was split), and the lower variance than appending without splits."""
    s = CONFIGS["tiny"].scaled(prefill=1024, n_clusters_init=24, var_alpha=1.2, size_factor=0.0, drift_std=0.15)
    w = generate(s, steps=512)
    K1, V1 = w["Knew"].transpose(1, 0, 2), w["Vnew"].transpose(1, 0, 2)          # the second chunk: drifted keys
    kw = dict(n_units=1, group_size=4, head_dim=128, n_clusters_init=24, max_clusters=512, max_tokens=1536, kmeans_iters=4,
              buffer_max=16, var_alpha=1.2)
    o = Oracle(OracleConfig(**kw))
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    o.extend(K1, V1)
    c, (off, mem) = o.clusters(0), o.members(0)
    assert o.num_tokens(0) == 1536 and sorted(mem.tolist()) == list(range(1536))
    assert c["flag"].sum() == 0 and c["b"].sum() == 0 and o.num_clusters(0) > 24 and o.diagnostics(0)["forced_splits"] == 0
    allK = np.concatenate([w["K0"][0], K1[0]]).astype(np.float64)
    for j in range(24, o.num_clusters(0)):                                        # children of splits: exact statistics
        m = mem[off[j]:off[j + 1]]
        np.testing.assert_allclose(c["centroids"][j], allK[m].mean(0), rtol=1e-5, atol=1e-6)
        assert c["M2"][j] == pytest.approx(((allK[m] - allK[m].mean(0)) ** 2).sum(), rel=1e-5, abs=1e-9)
    # the same entries through append + split with an empty active set but buffer_max = 0 give the same index
    p = Oracle(OracleConfig(**dict(kw, buffer_max=0)))
    p.build_index(w["K0"], w["V0"], w["init_idx"])
    for t in range(512):
        p.append(K1[:, t], V1[:, t]); p.split()
    np.testing.assert_array_equal(p.members(0)[1], mem)
    np.testing.assert_array_equal(p.clusters(0)["M2"], c["M2"])
    # static update of the same chunk leaves wider clusters
    q = Oracle(OracleConfig(**dict(kw, update_mode=1)))
    q.build_index(w["K0"], w["V0"], w["init_idx"])
    q.extend(K1, V1)
    cq = q.clusters(0)
    assert q.num_clusters(0) == 24 and c["M2"].sum() / 1536 < 0.8 * cq["M2"].sum() / 1536


def test_coretrieval_probabilities_and_placement_chain_on_a_hand_example():
    """Section 5.1, Eq. 8 by hand: three clusters of one entry each at (10,0), (0,10), (-10,0); budget 2 selects the
    two best clusters.  Queries (1,1) x2 -> {0,1}; (-1,1) -> {1,2}: f(0,1) = f(1,0) = 2, f(1,2) = f(2,1) = 1, sum 6;
    cluster 1 has the largest total (3), is co-retrieved most often with 0, then 2 is left: chain 1, 0, 2."""
    K = np.array([[10, 0], [0, 10], [-10, 0]], np.float32)[None]
    o = Oracle(cfg(M0=3, maxc=3, maxt=8, iters=1))
    o.build_index(K, K, np.array([[0, 1, 2]], np.int32))
    Q = np.array([[1, 1], [1, 1], [-1, 1]], np.float32)[:, None, None, :]
    P, order = o.coretrieval(Q, 2)
    want = np.zeros((3, 3))
    want[0, 1] = want[1, 0] = 2 / 6
    want[1, 2] = want[2, 1] = 1 / 6
    np.testing.assert_allclose(P[0], want, rtol=1e-15)
    assert order[0].tolist() == [1, 0, 2]
    assert P[0].sum() == pytest.approx(1.0)
    # no co-retrieval at all (budget for one cluster): zero matrix, chain by id
    P, order = o.coretrieval(Q, 1)
    assert P.sum() == 0 and order[0].tolist() == [0, 1, 2]


def test_local_update_clusters_each_window_of_new_entries_on_its_own():
    """update_mode = 3 (Section 2.3, local update): new entries stay clusters of their own until a window is full; its
    k-means (initial centres = every (W/k)-th entry) then replaces them by k clusters; the prefill's clusters never
    change.  The window's k-means against scikit-learn from the same centres."""
    from sklearn.cluster import KMeans
    s = CONFIGS["tiny"].scaled(prefill=400, n_clusters_init=10, drift_std=0.1)
    W, k, T = 48, 6, 4
    w = generate(s, steps=2 * W + 5)
    o = Oracle(OracleConfig(1, 4, 128, 10, 400, 400 + 2 * W + 5, T, 16, 0, 1.5, 2.0, 0.0, search_copy=1, update_mode=3,
                            local_window=W, local_clusters=k))
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    c0 = o.clusters(0)
    for t in range(2 * W + 5):
        o.retrieve_attend(w["Q"][t], 64)
        o.append(w["Knew"][t], w["Vnew"][t])
        o.split()
        done = (t + 1) // W
        assert o.num_clusters(0) == 10 + done * k + (t + 1) % W
    c, (off, mem) = o.clusters(0), o.members(0)
    for key in ("centroids", "n", "M2"):
        np.testing.assert_array_equal(c[key][:10], c0[key])                      # existing clusters are left alone
    assert c["flag"].sum() == 0 and sorted(mem.tolist()) == list(range(400 + 2 * W + 5))
    for win in range(2):
        X = w["Knew"][win * W:(win + 1) * W, 0].astype(np.float64)
        init = X[[j * W // k for j in range(k)]]
        full = KMeans(k, init=init, n_init=1, algorithm="lloyd", max_iter=T, tol=0).fit(X)
        prev = KMeans(k, init=init, n_init=1, algorithm="lloyd", max_iter=T - 1, tol=0).fit(X)
        ids = range(10 + win * k, 10 + (win + 1) * k)
        lab = np.full(W, -1)
        for j in ids:
            lab[mem[off[j]:off[j + 1]] - (400 + win * W)] = j - ids[0]
        np.testing.assert_array_equal(lab, prev.labels_)
        assert c["n"][list(ids)].min() > 0
        np.testing.assert_allclose(c["centroids"][list(ids)], full.cluster_centers_, rtol=1e-6, atol=1e-6)
        for j in ids:
            m = mem[off[j]:off[j + 1]] - (400 + win * W)
            assert c["M2"][j] == pytest.approx(((X[m] - c["centroids"][j].astype(np.float64)) ** 2).sum(), rel=1e-12)
    assert (c["n"][10 + 2 * k:] == 1).all()                                      # the open window: clusters of one


def test_imported_state_continues_like_the_original():
    s = CONFIGS["tiny"].scaled(var_alpha=1.2, buffer_max=4)
    w = generate(s, steps=96)
    kw = dict(n_units=1, group_size=4, head_dim=128, n_clusters_init=32, max_clusters=128, max_tokens=s.prefill + 96,
              kmeans_iters=3, buffer_max=4, var_alpha=1.2, size_factor=2.0)
    a = Oracle(OracleConfig(**kw))
    a.build_index(w["K0"], w["V0"], w["init_idx"])
    for t in range(48):
        a.retrieve_attend(w["Q"][t], 256); a.append(w["Knew"][t], w["Vnew"][t]); a.split()
    a.retrieve_attend(w["Q"][48], 256)            # the active set travels with the state
    b = Oracle(OracleConfig(**kw))
    c, (off, mem), (K, V) = a.clusters(0), a.members(0), a.kv(0)
    assert c["flag"].sum() > 0                    # the state carries flagged clusters and their buffers
    b.import_unit(0, K, V, c["centroids"], c["n"], c["b"], c["flag"], c["M2"], off, mem, a.tau(0), a.selected(0))
    for t in range(48, 96):
        if t > 48:
            oa, la = a.retrieve_attend(w["Q"][t], 256)
            ob, lb = b.retrieve_attend(w["Q"][t], 256)
            np.testing.assert_array_equal(oa, ob)
            np.testing.assert_array_equal(a.gather(0), b.gather(0))
        for o in (a, b):
            o.append(w["Knew"][t], w["Vnew"][t]); o.split()
    ca, cb = a.clusters(0), b.clusters(0)
    for k in ca:
        np.testing.assert_array_equal(ca[k], cb[k])
    np.testing.assert_array_equal(a.members(0)[1], b.members(0)[1])
    assert a.num_clusters(0) == b.num_clusters(0) > c["n"].shape[0]


# ---------------------------------------------------------------- decode properties on a realistic workload

@pytest.fixture(scope="module")
def tiny_run():
    s = CONFIGS["tiny"].scaled(var_alpha=1.2)
    w = generate(s)
    o = Oracle(OracleConfig(1, 4, 128, 32, 128, s.max_tokens, 10, 4, 0, s.var_alpha, s.size_factor, 0.0))
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    return s, w, o


def test_trajectory_invariants_and_split_partition(tiny_run):
    s, w, o = tiny_run
    allK = np.concatenate([w["K0"][0], w["Knew"][:, 0]]).astype(np.float64)
    n_split_seen = 0
    for t in range(s.steps):
        o.retrieve_attend(w["Q"][t], s.budget)
        sel, gat = o.selected(0), o.gather(0)
        off, mem = o.members(0)
        sizes = np.diff(off)
        assert sizes[sel].sum() == len(gat) <= s.budget
        sc = o.scores(0)
        rest = np.setdiff1d(np.arange(len(sc)), sel)
        assert len(rest) == 0 or sc[sel].min() >= sc[rest].max()             # a prefix of the score order
        o.append(w["Knew"][t], w["Vnew"][t])
        before = {j: mem[off[j]:off[j + 1]].tolist() for j in range(len(sizes))}
        j = o.last_assign(0)
        before[j] = before[j] + [s.prefill + t]
        M_before = o.num_clusters(0)
        o.split()
        c, (off, mem) = o.clusters(0), o.members(0)
        M = o.num_clusters(0)
        assert sorted(mem.tolist()) == list(range(s.prefill + t + 1))          # every token in exactly one cluster
        np.testing.assert_array_equal(np.diff(off), c["n"] + c["b"])
        assert np.all((c["b"] > 0) == (c["flag"] > 0))
        assert c["b"].sum() < 4 or M > M_before                               # buffers stay under B_max
        for new in range(M_before, M):                                         # children partition the parent
            parents = [p for p in before if set(mem[off[new]:off[new + 1]]) <= set(before[p])]
            assert len(parents) == 1
            p = parents[0]
            kid, stay = mem[off[new]:off[new + 1]].tolist(), mem[off[p]:off[p + 1]].tolist()
            assert sorted(kid + stay) == before[p] and kid == sorted(kid) and stay == sorted(stay)
            assert stay[0] == before[p][0]
            for jj in (p, new):                                               # exact statistics after a split
                m = mem[off[jj]:off[jj + 1]]
                np.testing.assert_allclose(c["centroids"][jj], allK[m].mean(0), rtol=2e-7, atol=1e-7)
                ss = ((allK[m] - c["centroids"][jj].astype(np.float64)) ** 2).sum()
                assert c["M2"][jj] == pytest.approx(ss, rel=1e-12, abs=1e-12)
            n_split_seen += 1
    assert n_split_seen == o.diagnostics(0)["splits"] > 0


def test_updatevar_is_the_two_pass_variance():
    s = CONFIGS["tiny"]
    w = generate(s)
    o = Oracle(OracleConfig(1, 4, 128, 32, 32, s.max_tokens, 10, 16, 0, 0.0, 0.0, 0.0))   # no trigger at all
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    for t in range(s.steps):
        o.append(w["Knew"][t], w["Vnew"][t])
    allK = np.concatenate([w["K0"][0], w["Knew"][:, 0]]).astype(np.float64)
    c, (off, mem) = o.clusters(0), o.members(0)
    assert c["flag"].sum() == 0 and c["n"].sum() == s.max_tokens
    for j in range(32):
        X = allK[mem[off[j]:off[j + 1]]]
        np.testing.assert_allclose(c["centroids"][j], X.mean(0), rtol=1e-5, atol=1e-6)
        assert c["M2"][j] == pytest.approx(((X - X.mean(0)) ** 2).sum(), rel=1e-6)


def test_full_budget_is_dense_attention_and_order_does_not_matter(tiny_run):
    s, w, _ = tiny_run
    rng = np.random.default_rng(7)
    K, V, Q = w["K0"][:, :512], w["V0"][:, :512], w["Q"][0]
    init = rng.choice(512, 16, replace=False).astype(np.int32)[None]
    o = Oracle(OracleConfig(1, 4, 128, 16, 16, 600, 4, 16, 0, 0.0, 0.0, 0.0))
    o.build_index(K, V, init)
    out, lse = o.retrieve_attend(Q, 512)
    assert len(o.selected(0)) == 16 and sorted(o.gather(0).tolist()) == list(range(512))
    ref, rl = dense_attention(Q[0], K[0], V[0], 1 / np.sqrt(128))
    np.testing.assert_allclose(out[0], ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(lse[0], rl, rtol=1e-12)
    # the same tokens in another order give the same attention; huge logits do not overflow
    perm = rng.permutation(512)
    o2 = Oracle(OracleConfig(1, 4, 128, 16, 16, 600, 4, 16, 0, 0.0, 0.0, 0.0))
    o2.build_index(K[:, perm], V[:, perm], init)
    out2, _ = o2.retrieve_attend(Q, 512)
    np.testing.assert_allclose(out2, out, rtol=1e-10, atol=1e-12)
    out3, lse3 = o.retrieve_attend(Q * 300, 512)
    assert np.isfinite(out3).all() and np.isfinite(lse3).all()
    # a partial retrieval equals dense attention restricted to the gathered tokens
    out4, lse4 = o.retrieve_attend(Q, 200)
    g = o.gather(0)
    assert 0 < len(g) <= 200
    ref, rl = dense_attention(Q[0], K[0][g], V[0][g], 1 / np.sqrt(128))
    np.testing.assert_allclose(out4[0], ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(lse4[0], rl, rtol=1e-12)


def test_scores_group_reduce_and_scale():
    rng = np.random.default_rng(8)
    X = rng.standard_normal((1, 64, 8)).astype(np.float32)
    Q = rng.standard_normal((1, 3, 8)).astype(np.float32)
    init = np.arange(5, dtype=np.int32)[None]
    for red in (0, 1):
        for scale in (0.0, 0.25):
            o = Oracle(cfg(G=3, d=8, M0=5, maxc=5, maxt=64, iters=2, reduce=red, scale=scale))
            o.build_index(X, X, init)
            o.retrieve_attend(Q, 10)
            S = Q[0].astype(np.float64) @ o.clusters(0)["centroids"].astype(np.float64).T
            want = (S.max(0) if red == 0 else S.sum(0)) * (scale or 1 / np.sqrt(8))
            np.testing.assert_allclose(o.scores(0), want, rtol=3e-7, atol=1e-7)


def test_selection_is_the_longest_fitting_prefix_brute_force():
    rng = np.random.default_rng(9)
    for trial in range(40):
        M = int(rng.integers(2, 8))
        X, _ = blobs(rng, 60, 4, M)
        init = rng.choice(60, M, replace=False).astype(np.int32)[None]
        o = Oracle(cfg(G=2, d=4, M0=M, maxc=M, maxt=60, iters=3))
        o.build_index(X[None], X[None], init)
        Q = rng.standard_normal((1, 2, 4)).astype(np.float32)
        sizes = o.clusters(0)["n"]
        prev = -1
        for B in range(1, 61, 3):
            o.retrieve_attend(Q, B)
            sc = o.scores(0)
            order = sorted(range(M), key=lambda j: (-sc[j], j))
            best = max(k for k in range(M + 1) if sizes[order[:k]].sum() <= B)   # try every prefix length
            sel, g = o.selected(0).tolist(), o.gather(0)
            if best == 0:
                off, mem = o.members(0)
                assert sel == order[:1] and g.tolist() == mem[off[sel[0]]:off[sel[0] + 1]][:B].tolist()
            else:
                assert sel == order[:best] and len(g) == sizes[sel].sum() <= B
            assert len(g) >= prev or best == 0
            prev = len(g)


def test_full_budget_splits_every_flagged_cluster_at_once_and_keeps_every_token():
    s = CONFIGS["tiny"].scaled(var_alpha=1.2)
    w = generate(s)
    runs = {}
    for name, bmax, budget in (("all_resident", 0, 64), ("full_budget", 16, 10 ** 6)):
        o = Oracle(OracleConfig(1, 4, 128, 32, 128, s.max_tokens, 10, bmax, 0, s.var_alpha, s.size_factor, 0.0))
        o.build_index(w["K0"], w["V0"], w["init_idx"])
        for t in range(s.steps):
            o.retrieve_attend(w["Q"][t], budget)
            o.append(w["Knew"][t], w["Vnew"][t])
            o.split()
            assert o.clusters(0)["flag"].sum() == 0
        runs[name] = o
    a, b = runs["all_resident"], runs["full_budget"]
    assert a.num_clusters(0) == b.num_clusters(0) > 32
    np.testing.assert_array_equal(a.labels(0), b.labels(0))


def test_capacity_errors_leave_state_consistent():
    g = json.load(open(os.path.join(GOLD, "hand_example_3_split.json")))
    K = np.array(g["keys"], np.float32)[None]
    o = Oracle(cfg(maxc=2, maxt=7, alpha=1.5, bmax=0))
    o.build_index(K, K, np.array([g["init_idx"]], np.int32))
    k = np.array([g["new_key"]], np.float32)
    o.append(k, k); o.split()
    assert o.num_clusters(0) == 2 and o.error(0) == 2 and o.clusters(0)["flag"][0] == 1
    o.append(k, k)
    assert o.num_tokens(0) == 7 and o.error(0) == 3
    with pytest.raises(ValueError):
        Oracle(cfg(maxt=4)).build_index(K, K, np.array([[0, 4]], np.int32))


# ---------------------------------------------------------------- search copies in the storage type

def _bf16(x):
    u = np.asarray(x, np.float32).view(np.uint32)
    return ((u + (((u >> 16) & 1) + 0x7FFF)) & np.uint32(0xFFFF0000)).view(np.float32)


def test_storage_rounding_is_ieee_round_to_nearest_even():
    from oracle import round_to_storage
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(100000) * 10.0 ** rng.integers(-9, 5, 100000)).astype(np.float32)
    x = np.concatenate([x, np.array([0, -0.0, 65504, 65519.99, 65520, 7e4, 1e-8, 2 ** -25, 2 ** -24, 3e-8, -6.1e-5,
                                     2049, 2051, 1 + 2 ** -11, 1 + 3 * 2 ** -11], np.float32)])
    with np.errstate(over="ignore"):
        np.testing.assert_array_equal(round_to_storage(x, "f16"), x.astype(np.float16).astype(np.float32))
    np.testing.assert_array_equal(round_to_storage(x, "bf16"), _bf16(x))
    np.testing.assert_array_equal(round_to_storage(x, "f32"), x)
    assert round_to_storage(np.float32([2049.0]), "f16")[0] == 2048.0      # tie -> even
    assert round_to_storage(np.float32([2051.0]), "f16")[0] == 2052.0


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_searches_read_the_centroids_in_the_storage_type(dtype):
    """Scores and nearest-cluster assignment use r_j rounded to the storage type; the float32 mean itself and the
    statistics do not change.  Checked against numpy on a drifting trajectory with appends and splits."""
    s = CONFIGS["tiny"].scaled(dtype=dtype, var_alpha=1.2, size_factor=0.0, buffer_max=4)
    w = generate(s, steps=96)
    o = Oracle(OracleConfig(1, 4, 128, 32, 128, s.max_tokens, 5, 4, 0, s.var_alpha, 0.0, 0.0, dtype=dtype))
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    conv = (lambda a: a.astype(np.float16).astype(np.float32)) if dtype == "f16" else _bf16
    differ = 0
    for t in range(96):
        c = o.clusters(0)
        rs = o.search_copy(0)
        np.testing.assert_array_equal(rs, conv(c["centroids"]))
        q = w["Q"][t, 0].astype(np.float64)
        o.retrieve_attend(w["Q"][t], 256)
        want = (q @ rs.astype(np.float64).T).max(0) / np.sqrt(128)
        got = o.scores(0)
        np.testing.assert_allclose(got, want, rtol=2e-7, atol=1e-30)
        plain = ((q @ c["centroids"].astype(np.float64).T).max(0) / np.sqrt(128)).astype(np.float32)
        differ += int((got != plain).sum())
        k = w["Knew"][t, 0].astype(np.float64)
        d2 = ((k[None, :] - rs.astype(np.float64)) ** 2).sum(1)
        o.append(w["Knew"][t], w["Vnew"][t])
        order = np.argsort(d2, kind="stable")
        if len(order) == 1 or d2[order[1]] - d2[order[0]] > 1e-9 * d2[order[0]]:
            assert o.last_assign(0) == order[0]
        o.split()
    assert differ > 0          # the rounding is visible: scores are not those of the unrounded means
    assert o.diagnostics(0)["splits"] > 0


def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """oracle/sanitize_check.cpp drives every call of the oracle (prefill, retrievals, appends, delayed and forced
    splits, a state import, the capacity limits) in a build with -fsanitize=address,undefined."""
    import subprocess
    src = os.path.join(os.path.dirname(GOLD), "..", "oracle", "sanitize_check.cpp")
    exe = str(tmp_path / "sanitize_check")
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fopenmp", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", src, "-o", exe])
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                       env=dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0", OMP_NUM_THREADS="2"))
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitize_check ok" in r.stdout
