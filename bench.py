"""Benchmark of the decode hot path on one MI355X.

A step = dynakv_decode_step (retrieve + attend, append, split) over all units of the workload, on seeded
synthetic drifting-mixture inputs already resident in HBM.  Prints one JSON line: decode steps/s, the
roofline of the dominant kernel (the whole step in one launch where the shape allows: scores, selection, append,
gather + attention, splits; else gather + attention; HBM-bound), and the CPU oracle timed on a bounded sample
of the same workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0      # dense fp16/bf16, published

# HBM bytes per launch of the dominant kernel from two `rocprofv3 --pmc` runs of this file (FETCH_SIZE, then
# WRITE_SIZE, KiB per dispatch averaged over the timed launches), each scaled by what the same counter reads for
# torch's float32 -> float16 conversion of the 134 217 728-element prefill keys in the same run (512 MiB read,
# 256 MiB written).  Keyed by (config, steps, warmup, units); "rev" is kernel_revision() of the sources the
# counters were taken with: another revision of the kernels, or other arguments, report null.
PMC_TRAFFIC = {
    ("llama3_8b", 8192, 64, 0): {"rev": "1035b3543096", "kernel": "retrieve_fused_kernel", "fetch_kib": 111299.5,
                                 "fetch_scale": 524288.0 / 262168.94, "write_kib": 4661.7, "write_scale": 262144.0 / 262144.0},
    ("llama3_8b", 20, 5, 0): {"rev": "1035b3543096", "kernel": "retrieve_fused_kernel", "fetch_kib": 85354.7,
                              "fetch_scale": 524288.0 / 262170.0, "write_kib": 2379.3, "write_scale": 262144.0 / 262144.0},
}


def kernel_revision() -> str:
    """First 12 hex digits of the SHA-256 over the kernel sources: ties measured counters to the code they measured."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2511_07427_amd", "csrc")
    for f in sorted(os.listdir(d)):
        with open(os.path.join(d, f), "rb") as fh:
            h.update(f.encode() + b"\0" + fh.read())
    return h.hexdigest()[:12]


def _oracle_run(spec, n_units, steps, budget, threads):
    import numpy as np
    from oracle import Oracle, OracleConfig
    from paper_2511_07427_amd.workload import generate
    w = generate(spec, units=range(n_units), steps=steps)
    o = Oracle(OracleConfig(n_units, spec.group_size, spec.head_dim, spec.n_clusters_init, spec.max_clusters,
                            spec.prefill + steps, spec.kmeans_iters, spec.buffer_max, 0, spec.var_alpha,
                            spec.size_factor, 0.0, dtype=spec.dtype), threads=threads)
    t0 = time.perf_counter()
    o.build_index(w["K0"], w["V0"], w["init_idx"])
    t1 = time.perf_counter()
    for t in range(steps):
        o.retrieve_attend(w["Q"][t], budget)
        o.append(w["Knew"][t], w["Vnew"][t])
        o.split()
    t2 = time.perf_counter()
    return t1 - t0, t2 - t1, o.threads_used


def cpu_baseline(spec, budget):
    """The oracle as it stands on bounded samples of the same workload: k-means prefill plus decode steps of the
    first units, once on all host threads and once on one; the rates are scaled to all units of the workload."""
    cores = os.cpu_count() or 1
    nu = min(spec.n_units, 32)
    steps = 1536
    pre, dec, used = _oracle_run(spec, nu, steps, budget, 0)
    nu1, steps1 = min(spec.n_units, 2), 384
    pre1, dec1, _ = _oracle_run(spec, nu1, steps1, budget, 1)
    return dict(value=steps / (dec * spec.n_units / nu), unit="decode steps/s", cores=used, kind="oracle",
                sample="%d of %d units, %d-token k-means prefill (%.1f s, not in value) then %d decode steps in %.1f s on %d "
                       "threads; 1 thread: %d units, %d steps in %.1f s; rates scaled to all units" %
                       (nu, spec.n_units, spec.prefill, pre, steps, dec, used, nu1, steps1, dec1),
                value_1_thread=steps1 / (dec1 * spec.n_units / nu1), host_threads=cores,
                prefill_s_all_units=pre * spec.n_units / nu, prefill_s_all_units_1_thread=pre1 * spec.n_units / nu1)


def variants_report(a):
    """The update strategies the paper compares (Section 2.3, Section 8.1, Table 5) on the same drifting workload and
    kernels: adaptive (Algorithm 1), static update (append to the nearest cluster, never split), local update (new
    entries clustered among themselves, window by window) and no clustering (every entry its own cluster: exact
    top-B over tokens).  Per strategy: decode steps/s, recall of the dense top-B
    tokens, share of the dense attention mass that the retrieved entries carry, error of the attention output
    against dense attention, mean intra-cluster variance, clusters per unit.  Quality is sampled every
    `--variant-every` steps through the three-call API (the gather list is read back before the split)."""
    import numpy as np
    import torch
    from paper_2511_07427_amd import binding
    from paper_2511_07427_amd.workload import CONFIGS, generate
    base = CONFIGS[a.config].scaled(n_units=a.units or 32)
    T, every = a.steps, a.variant_every
    dev = torch.device("cuda:0")
    tdt = binding.TORCH_DTYPES[base.dtype]
    w = generate(base, steps=T, workers=16)
    K0, V0 = torch.from_numpy(w["K0"]).to(dev).to(tdt), torch.from_numpy(w["V0"]).to(dev).to(tdt)
    Q, Kn, Vn = (torch.from_numpy(w[k]).to(dev).to(tdt) for k in ("Q", "Knew", "Vnew"))
    U, G, d, B = base.n_units, base.group_size, base.head_dim, base.budget
    scale = 1.0 / np.sqrt(d)
    out, lse = torch.empty(U, G, d, device=dev), torch.empty(U, G, device=dev)
    res = {}
    LW, LK = 64, 32                       # local update: windows of 64 entries into 32 clusters (many small clusters)
    for name, mode in (("adaptive", binding.UPDATE_ADAPTIVE), ("static", binding.UPDATE_STATIC), ("local", binding.UPDATE_LOCAL),
                       ("tokens", binding.UPDATE_TOKENS)):
        tok, loc = mode == binding.UPDATE_TOKENS, mode == binding.UPDATE_LOCAL
        M0 = base.prefill if tok else base.n_clusters_init
        Mcap = base.prefill + T if tok else base.n_clusters_init + LW + LK * (T // LW + 1) if loc else base.max_clusters
        ix = binding.Index(binding.Config(U, G, base.dtype, M0, Mcap, base.prefill + T, 1 if tok else base.kmeans_iters,
                                          base.buffer_max, 0, base.var_alpha, base.size_factor, 0.0, update_mode=mode,
                                          local_window=LW if loc else 0, local_clusters=LK if loc else 0), dev)
        init = torch.arange(base.prefill, dtype=torch.int32, device=dev).repeat(U, 1) if tok else torch.from_numpy(w["init_idx"]).to(dev)
        ix.dynakv_build_index(K0, V0, init.contiguous())
        torch.cuda.synchronize()
        recall, mass, err, busy = [], [], [], 0.0
        for t in range(T):
            if t % every == every - 1:
                ix.dynakv_retrieve_attend(Q[t], B, out, lse)
                st = ix.dynakv_export_state(["n_gathered", "gathered", "n_tokens", "keys", "values"], to_cpu=False)
                N = int(st["n_tokens"][0])
                Kf, Vf, qf = st["keys"][:, :N].float(), st["values"][:, :N].float(), Q[t].float()
                logit = torch.einsum("ugd,und->ugn", qf, Kf) * scale
                p = torch.softmax(logit, -1)
                dense = torch.einsum("ugn,und->ugd", p, Vf)
                sel = torch.zeros(U, N, device=dev)
                for u in range(U):
                    sel[u, st["gathered"][u, :int(st["n_gathered"][u])].long()] = 1.0
                top = logit.max(1).values.topk(min(B, N), -1).indices
                recall.append(float(sel.gather(1, top).mean()))
                mass.append(float((p * sel[:, None, :]).sum(-1).mean()))
                err.append(float(((out - dense).norm(dim=-1) / dense.norm(dim=-1).clamp_min(1e-6)).mean()))
                ix.dynakv_append(Kn[t], Vn[t])
                ix.dynakv_split()
                torch.cuda.synchronize()
            else:
                t0 = time.perf_counter()
                ix.dynakv_decode_step(Q[t], B, out, lse, Kn[t], Vn[t])
                if t % every == every - 2:
                    torch.cuda.synchronize()
                busy += time.perf_counter() - t0
        torch.cuda.synchronize()
        st = ix.dynakv_export_state(["n_clusters", "size", "m2", "error"])
        n, m2 = st["size"].double().sum(), st["m2"].sum()
        res[name] = dict(steps_per_s=(T - T // every) / busy, recall_of_dense_top_b=float(np.mean(recall)),
                         dense_attention_mass_retrieved=float(np.mean(mass)), attention_error_vs_dense=float(np.mean(err)),
                         mean_cluster_variance=float(m2 / n), clusters_per_unit=float(st["n_clusters"].float().mean()),
                         error_words=int(st["error"].abs().sum()))
        print("[bench] %s: %s" % (name, res[name]), file=sys.stderr, flush=True)
        del ix
    print(json.dumps({"metric": "update strategies on the same drifting workload", "n_gpus": 1, "steps": T, "data": "synthetic",
                      "config": {"workload": "%s shape, %d units, prefill %d, budget %d, %d decode steps, quality sampled every %d steps"
                                             % (base.name, U, base.prefill, B, T, every)},
                      "variants": res}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8192)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--config", default="llama3_8b")
    ap.add_argument("--units", type=int, default=0,
                    help="run UNITS units instead of the configuration's own count: fewer = its first units; more = "
                         "further independent draws of the same shape (more layers or sequences), labelled as such")
    ap.add_argument("--max-cluster-factor", type=int, default=0,
                    help="max_clusters = FACTOR x the initial cluster count instead of the configuration's own factor "
                         "(long runs whose drift needs more clusters; above 4096 clusters the separate kernels run)")
    ap.add_argument("--full-horizon", action="store_true",
                    help="run the configuration to the end of its own decode length (steps = that length minus the "
                         "warm-up) with the cluster capacity such a run needs")
    ap.add_argument("--variants", action="store_true",
                    help="instead of the benchmark line: adaptive, static-update and token-level retrieval on the same "
                         "workload (default 32 units), with recall, attention error and cluster variance")
    ap.add_argument("--variant-every", type=int, default=128)
    ap.add_argument("--coretrieval-refs", type=int, default=0,
                    help="after the prefill, lay the pages out by co-retrieval (dynakv_place_by_coretrieval) with the "
                         "first N queries as the reference input")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true", help="skip the HIP events around the dominant kernel")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this path runs on one GPU; units (layer, sequence, KV head) are independent and would "
                 "shard over GPUs without communication, but no multi-GPU run exists here. Use --gpus 1.")

    if a.variants:
        return variants_report(a)

    import numpy as np
    import torch
    from paper_2511_07427_amd import binding
    from paper_2511_07427_amd.workload import CONFIGS, generate

    from paper_2511_07427_amd.workload import FULL_HORIZON_FACTOR
    spec = CONFIGS[a.config]
    if a.full_horizon:
        a.steps = spec.steps - a.warmup
        spec = spec.scaled(max_cluster_factor=FULL_HORIZON_FACTOR[a.config])
    own_units = spec.n_units
    if a.units:
        spec = spec.scaled(n_units=a.units)
    if a.max_cluster_factor:
        spec = spec.scaled(max_cluster_factor=a.max_cluster_factor)
    T = a.warmup + a.steps
    U, G, d = spec.n_units, spec.group_size, spec.head_dim
    dev = torch.device("cuda:0")
    tdt = binding.TORCH_DTYPES[spec.dtype]
    esz = 4 if spec.dtype == "f32" else 2

    def say(msg):                      # progress on stderr: long runs must not look hung
        print("[bench] " + msg, file=sys.stderr, flush=True)

    t0 = time.perf_counter()
    w = generate(spec, steps=T, workers=16)
    gen_s = time.perf_counter() - t0
    say("inputs generated in %.1f s" % gen_s)
    K0 = torch.from_numpy(w["K0"]).to(dev).to(tdt)
    V0 = torch.from_numpy(w["V0"]).to(dev).to(tdt)
    init = torch.from_numpy(w["init_idx"]).to(dev)
    Q = torch.empty(T, U, G, d, dtype=tdt, device=dev)
    Kn = torch.empty(T, U, d, dtype=tdt, device=dev)
    Vn = torch.empty(T, U, d, dtype=tdt, device=dev)
    for lo in range(0, T, 512):           # staged upload keeps the float32 host copies off the device
        hi = min(T, lo + 512)
        Q[lo:hi] = torch.from_numpy(w["Q"][lo:hi]).to(dev).to(tdt)
        Kn[lo:hi] = torch.from_numpy(w["Knew"][lo:hi]).to(dev).to(tdt)
        Vn[lo:hi] = torch.from_numpy(w["Vnew"][lo:hi]).to(dev).to(tdt)
    del w
    say("inputs resident in HBM")

    ix = binding.Index(binding.Config(U, G, spec.dtype, spec.n_clusters_init, spec.max_clusters, spec.prefill + T,
                                      spec.kmeans_iters, spec.buffer_max, 0, spec.var_alpha, spec.size_factor, 0.0), dev)
    out = torch.empty(U, G, d, dtype=torch.float32, device=dev)
    lse = torch.empty(U, G, dtype=torch.float32, device=dev)
    st = torch.cuda.current_stream()
    stream = st.cuda_stream

    # prefill (one-off, reported beside the decode figure)
    ix.dynakv_build_index(K0, V0, init)          # first call also pays module loading
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    ix.dynakv_build_index(K0, V0, init)
    e1.record(st)
    torch.cuda.synchronize()
    prefill_ms = e0.elapsed_time(e1)
    # the same prompt through chunked prefill: k-means on the first half, adaptive extension with the second half
    half = spec.prefill // 2
    Ka, Va, Kb, Vb = (x.contiguous() for x in (K0[:, :half], V0[:, :half], K0[:, half:], V0[:, half:]))
    chunked = None
    if spec.n_clusters_init <= half:
        init_half = (torch.arange(spec.n_clusters_init, dtype=torch.int32, device=dev) * (half // spec.n_clusters_init)).repeat(U, 1).contiguous()
        ix.dynakv_build_index(Ka, Va, init_half)
        e0.record(st)
        ix.dynakv_extend_index(Kb, Vb)
        e1.record(st)
        torch.cuda.synchronize()
        sx = ix.dynakv_export_state(["n_clusters", "error"])
        chunked = {"extend_ms": e0.elapsed_time(e1), "tokens_per_unit": spec.prefill - half,
                   "tokens_per_s_all_units": (spec.prefill - half) * U / (e0.elapsed_time(e1) * 1e-3),
                   "clusters_mean_after": float(sx["n_clusters"].float().mean()), "error_words": int(sx["error"].abs().sum())}
    ix.dynakv_build_index(K0, V0, init)          # back to the index the decode steps start from
    if a.coretrieval_refs:
        ix.dynakv_place_by_coretrieval(K0, V0, Q[:a.coretrieval_refs].contiguous(), spec.budget)
    torch.cuda.synchronize()
    kmeans_flop = 2.0 * spec.prefill * spec.n_clusters_init * d * spec.kmeans_iters * U

    qs, ks, os_, ls = Q.data_ptr(), Kn.data_ptr(), out.data_ptr(), lse.data_ptr()
    q_stride, k_stride = U * G * d * esz, U * d * esz
    step = ix.decode_step_ptrs
    say("prefill %.2f ms" % prefill_ms)
    for t in range(a.warmup):
        step(qs + t * q_stride, spec.budget, os_, ls, ks + t * k_stride, Vn.data_ptr() + t * k_stride, stream)
        if t % 8192 == 8191:
            torch.cuda.synchronize()
            say("warm-up step %d" % (t + 1))
    torch.cuda.synchronize()
    c0 = ix.dynakv_export_state(["counters"])["counters"].numpy().copy()
    # HIP events around a launch put several microseconds between two kernels of the stream and a few into what they
    # measure, so an even sample of the timed launches is bracketed: of every 16 launches the first 4 inside one pair
    # of events where the step is one kernel (of a 20-step run: 2 x 5), else every 16th launch alone
    one_kernel = ix.dynakv_profiled_kernel() == "retrieve_fused_kernel"
    every = max(1, min(16, a.steps // 2))
    run = max(1, min(4 if a.steps >= 64 else 5, every // 2)) if one_kernel else 1
    brackets = a.steps // every + (1 if a.steps % every >= run else 0)
    timed_launches = brackets * run
    if not a.no_kernel_events:
        ix.dynakv_profile_sample(every, run)
        ix.dynakv_profile_enable(brackets)
    vs = Vn.data_ptr()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(a.warmup, T):
        step(qs + t * q_stride, spec.budget, os_, ls, ks + t * k_stride, vs + t * k_stride, stream)
        if (t & 16383) == 16383:
            say("enqueued step %d" % (t + 1))           # no synchronisation inside the timed region
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    state = ix.dynakv_export_state(["counters", "error", "n_clusters", "n_tokens"])
    c1 = state["counters"].numpy()
    if int(state["error"].abs().sum()) != 0:
        bad = state["error"].nonzero().flatten().tolist()
        sys.exit("bench.py: device error word set: units %s bits %s clusters %s tokens %s" %
                 (bad[:8], state["error"][bad[:8]].tolist(), state["n_clusters"][bad[:8]].tolist(),
                  state["n_tokens"][bad[:8]].tolist()))
    assert int(state["n_tokens"].min()) == spec.prefill + T
    gathered = int((c1[:, 4] - c0[:, 4]).sum())
    retrievals = int((c1[:, 5] - c0[:, 5]).sum())
    scored = int((c1[:, 6] - c0[:, 6]).sum())
    assert retrievals == a.steps * U

    roof = None
    if not a.no_kernel_events:
        n, ms = ix.dynakv_profile_read()
        assert n == timed_launches
        kernel = ix.dynakv_profiled_kernel()
        kv_bytes = gathered / a.steps * 2 * d * esz                    # K and V of every gathered entry, once
        centroid_bytes = scored / a.steps * d * esz if kernel == "retrieve_fused_kernel" else 0.0   # search copy in the storage type, once
        bytes_per_launch = kv_bytes + centroid_bytes
        achieved = bytes_per_launch / (ms / n * 1e-3) / 1e9
        pmc = PMC_TRAFFIC.get((a.config, a.steps, a.warmup, a.units))
        if pmc and (pmc["rev"] != kernel_revision() or pmc["kernel"] != kernel or a.max_cluster_factor or a.full_horizon or
                    a.coretrieval_refs):
            pmc = None
        traffic = (pmc["fetch_kib"] * pmc["fetch_scale"] + pmc["write_kib"] * pmc["write_scale"]) * 1024.0 if pmc else None
        roof = dict(bound="hbm", kernel=kernel, achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=achieved / HBM_PEAK_GBS, traffic=traffic, kernel_rev=kernel_revision(), avg_launch_us=ms / n * 1e3,
                    launches_timed=n, timed_every=every, launches_per_bracket=run,
                    algorithmic_bytes_per_launch=bytes_per_launch, kv_bytes_per_launch=kv_bytes,
                    centroid_bytes_per_launch=centroid_bytes, gathered_entries_per_unit=gathered / retrievals,
                    clusters_per_unit=scored / retrievals)

    res = {
        "metric": "decode steps/sec (index maint + retrieve + sparse attn)", "value": a.steps / dt,
        "unit": "decode steps/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt / a.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": spec.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d units (layers x KV heads)%s, G=%d, d=%d, %s, prefill %d, M0=%d clusters, "
                               "token budget %d, at most %d clusters, decode steps %d..%d of a drifting %d-component mixture" %
                               (spec.name, U, "" if U == own_units else " INSTEAD OF THE CONFIGURATION'S %d" % own_units,
                                G, d, spec.dtype, spec.prefill, spec.n_clusters_init, spec.budget, spec.max_clusters,
                                a.warmup, T, spec.n_components),
                   "coretrieval_refs": a.coretrieval_refs},
        "roofline": roof,
        "prefill": {"ms": prefill_ms, "kmeans_algorithmic_tflops": kmeans_flop / (prefill_ms * 1e-3) / 1e12,
                    "frac_of_mfma_peak": kmeans_flop / (prefill_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                    # the other bound of the k-means (it applies below about 312 initial clusters): every iteration
                    # must read the keys once
                    "frac_of_hbm_peak": spec.kmeans_iters * U * spec.prefill * d * esz / (prefill_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "chunked_second_half": chunked},
        "index": {"clusters_mean": float(state["n_clusters"].float().mean()), "clusters_max": int(state["n_clusters"].max()),
                  "splits": int(c1[:, 0].sum()),
                  "forced_splits": int(c1[:, 2].sum()), "input_generation_s": gen_s},
    }
    if not a.no_cpu_baseline:
        say("timing the oracle on the host")
        res["cpu_baseline"] = cpu_baseline(spec, spec.budget)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
