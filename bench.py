#!/usr/bin/env python3
"""Benchmark of the RetrievalAttention decode hot path on one MI355X.

Workload (default): the 128K-context decode configuration the headline metric is quoted on:
a Llama-3-8B-shaped model (Table 6: 32 layers, 32 query heads over 8 KV heads, d = 128), one
sequence, bf16 KV, N = 131072 keys and M = 131072 prefill queries per head, graph degree 32,
knn 32, topk 100, ef 256, sink 4 + window 640. One "step" = one generated token = 32
sequential per-layer decode-step attention calls (search, sparse + static attention, merge)
with all KV and graphs resident in HBM. Index build (exact KNN on the matrix cores +
projection) runs before the timed region and is reported separately.

Prints ONE JSON line: the metric and its value, the workload, `roofline` (the fused decode
kernel's algorithmic bytes per launch over its measured launch time, against 8 TB/s, with the
HBM traffic the counters read for this build of the kernel, if a summary under profiles/ has it),
`hbm_measured` (what a 1 GiB device copy, a read-only streaming kernel and a gather of scattered 256-byte
rows sustain on this device),
`stages`, `exact_baselines`, `build` (with `knn_kernel`: the index-build GEMM's live time for one
layer against the dense MFMA peak), `other_configs` (the batched and the 1M-key configurations,
measured the same way after the headline one), `cpu_baseline` (the oracle over the host's cores).
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0
MFMA_F32_PEAK_TFLOPS = 157.3
METRIC = "decode-step retrieval-attention latency (ms) @128K ctx, 1 GPU; recall@100"
# start-set size and expansion width per workload (the walk's own parameters; ef, topk, deg and knn
# are the workload's): the fastest setting of a sweep over (seeds, expand) that keeps recall@k where the
# single-entry walk had it or above
DEFAULT_SEEDS = {"config2": 2048, "config1": 1024, "config3": 1024, "config4": 2048, "config0": 0}
DEFAULT_EXPAND = {"config2": 256, "config1": 128, "config3": 64, "config4": 64, "config0": 64}
# sources that make up decode_kernel: a counter summary under profiles/ applies to this build
# only if it was taken with the same ones
DECODE_SOURCES = ["decode.hip", "search_dev.h", "attend_dev.h", "common.h"]


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=3)
    p.add_argument("--workload", default="config2",
                   choices=["config2", "config1", "config3", "config0", "config4"])
    p.add_argument("--layers", type=int, default=None, help="override the layer count (debug)")
    p.add_argument("--context", type=int, default=None, help="override N (debug)")
    p.add_argument("--seqs", type=int, default=None, help="config3: number of sequences (default 16)")
    p.add_argument("--topk", type=int, default=None, help="override the retrieval size (e.g. 2000)")
    p.add_argument("--ef", type=int, default=None, help="override the beam width")
    p.add_argument("--deg", type=int, default=None, help="override the graph degree (config2)")
    p.add_argument("--knn", type=int, default=None, help="override the KNN list length (config2)")
    p.add_argument("--expand", type=int, default=None, help="search expansion width (default per workload)")
    p.add_argument("--seeds", type=int, default=None,
                   help="start-set size of the walk (RA_CFG_SEEDS; 0: single entry point; default per workload)")
    p.add_argument("--tokens", type=int, default=8, help="distinct decode queries per head")
    p.add_argument("--recall-layers", type=int, default=2)
    p.add_argument("--cpu-heads", type=int, default=32, help="heads the CPU oracle is timed on")
    p.add_argument("--cpu-tokens", type=int, default=8, help="decode queries per head the CPU oracle is timed on")
    p.add_argument("--cpu-workers", type=int, default=16, help="host processes the CPU oracle is spread over")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-other-configs", action="store_true",
                   help="skip the batched (config3) and 1M-key (config4) measurements after the headline one")
    p.add_argument("--graph", type=int, default=1, help="replay the step from a captured HIP graph")
    p.add_argument("--q8", type=int, default=0,
                   help="1: the graph walk reads an 8-bit copy of the keys (ra_decode_step_q8)")
    p.add_argument("--seed-shares", type=int, default=None,
                   help="workgroups a head's start set is scored by beside its own (RA_CFG_SEED_SHARES: 0, 2..8; "
                        "default: the library's)")
    p.add_argument("--helpers", type=int, default=1,
                   help="0: every head attends to the static set itself (no helper workgroups)")
    p.add_argument("--copy-calibration", action="store_true",
                   help="also run three plain 1 GiB device copies (reference for HBM counters)")
    return p.parse_args()


def decode_sources_sha():
    h = hashlib.sha256()
    for f in DECODE_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2409_10516_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def traffic_from_profiles(workload, seeds, ef, expand):
    """HBM bytes per decode_kernel launch from a rocprofv3 counter summary under profiles/ (lines
    `bench_traffic: {json}`), if one was taken for this workload and walk and with this build of
    the kernel's sources; else None."""
    sha = decode_sources_sha()
    pdir = os.path.join(ROOT, "profiles")
    for name in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        for line in open(os.path.join(pdir, name), errors="replace"):
            m = re.match(r"\s*bench_traffic:\s*(\{.*\})\s*$", line)
            if not m:
                continue
            try:
                rec = json.loads(m.group(1))
            except ValueError:
                continue
            if (rec.get("workload"), rec.get("seeds"), rec.get("ef"), rec.get("expand"),
                    rec.get("kernel_sources_sha")) == (workload, seeds, ef, expand, sha):
                return rec.get("bytes_per_launch")
    return None


def _oracle_worker(job):
    """One (head, token list) share of the CPU baseline, in a host process of its own: the oracle's
    decode step on arrays mapped from /dev/shm. Returns (head, seconds of work, ids of the first token)."""
    import numpy as np
    from oracle import decode as OD
    (h, kvh, tokens, shm, sink, window, topk, ef, expand, n_seeds) = job
    K = np.load(os.path.join(shm, f"K{kvh}.npy"), mmap_mode="r")
    V = np.load(os.path.join(shm, f"V{kvh}.npy"), mmap_mode="r")
    adj = np.load(os.path.join(shm, f"adj{h}.npy"), mmap_mode="r")
    qs = np.load(os.path.join(shm, "q.npy"), mmap_mode="r")
    ent = int(np.load(os.path.join(shm, "entry.npy"))[h])
    t0 = time.perf_counter()
    first = None
    for t in tokens:
        _, _, ids, _ = OD.decode_step(qs[t, 0, h], K, V, adj, ent, sink, window, topk, ef, expand,
                                      n_seeds=n_seeds)
        if first is None:
            first = ids
    return h, time.perf_counter() - t0, first


def cpu_baseline(ra, L, n_q, n_kv, tokens, workers, sink, window, topk, ef, expand, n_seeds, heads, n_layers):
    """The oracle's decode step for a sample of heads of layer 0, spread over `workers` host processes
    (one index per process at a time, the paper's own CPU scheme of Appendix C), wall-clock timed."""
    import multiprocessing as mp
    import shutil
    import tempfile
    import numpy as np
    shm = tempfile.mkdtemp(prefix="ra_bench_", dir="/dev/shm" if os.path.isdir("/dev/shm") else None)
    try:
        G = n_q // n_kv
        n_cpu = len(heads)
        for kvh in sorted({h // G for h in heads}):
            np.save(os.path.join(shm, f"K{kvh}.npy"), L["K"][0, kvh].float().cpu().numpy())
            np.save(os.path.join(shm, f"V{kvh}.npy"), L["V"][0, kvh].float().cpu().numpy())
        ents = np.zeros(n_q, np.int32)
        for h in heads:
            adj, ent = ra.ra_index_export(L["idx"], 0, h)
            np.save(os.path.join(shm, f"adj{h}.npy"), adj.numpy())
            ents[h] = ent
        np.save(os.path.join(shm, "entry.npy"), ents)
        np.save(os.path.join(shm, "q.npy"), L["q"].float().cpu().numpy())
        jobs = [(h, h // G, tokens, shm, sink, window, topk, ef, expand, n_seeds) for h in heads]
        workers = max(1, min(workers, len(jobs)))
        ctx = mp.get_context("spawn")                 # the parent holds a GPU context: never fork it
        with ctx.Pool(workers) as pool:
            pool.map(time.sleep, [0.01] * workers)    # processes up, numpy and the oracle imported on first job
            t0 = time.perf_counter()
            res = pool.map(_oracle_worker, jobs, chunksize=1)
            wall = time.perf_counter() - t0
        work = sum(r[1] for r in res)
        return {h: ids for h, _, ids in res}, wall, work, workers
    finally:
        shutil.rmtree(shm, ignore_errors=True)


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards without exchange over "
              "layers, heads and sequences). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2409_10516_amd as ra
    from paper_2409_10516_amd import binding as B, synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    ra.lib()                                    # fail loudly if the HIP library is missing
    f32 = dict(dtype=torch.float32, device=dev)

    def log(msg):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    # ---- one workload: build, time the decode step, count the algorithmic bytes -------------------
    def measure(workload, steps, warmup, tokens, n_layers=None, context=None, seqs=None, topk=None, ef=None,
                deg=None, knn=None, expand=None, seeds=None, full=False):
        """-> (result dict, state for the extra measurements of the headline workload)."""
        expand = DEFAULT_EXPAND[workload] if expand is None else expand
        seeds = DEFAULT_SEEDS[workload] if seeds is None else seeds
        if workload == "config2":
            nl, N, n_seq = 32, 131072, 1
            kw = {k: v for k, v in (('deg', deg), ('knn', knn)) if v}
            mk = lambda l: synth.make_config2_layer(l, device=dev, N=N, T=tokens, **kw)
        elif workload == "config1":
            nl, N, n_seq = 1, 32768, 1
            mk = lambda l: synth.make_config1(device=dev, N=N, T=tokens)
        elif workload == "config3":
            nl, N, n_seq = 1, 32768, seqs or 16
            mk = lambda l: synth.make_config3(device=dev, N=N, T=tokens, n_seq=n_seq)
        elif workload == "config4":
            nl, N, n_seq = 1, 1 << 20, 1
            mk = lambda l: synth.make_config4(device=dev, N=N, T=tokens)
        else:
            nl, N, n_seq = 1, 4096, 1
            mk = lambda l: synth.make_config0(device=dev)
        if context:
            N = context
        nl = n_layers or nl
        layers = []
        t_gen = t_build = 0.0
        build_flop = 0.0
        knn_rec = None
        for l in range(nl):
            t0 = time.time()
            w = mk(l)
            torch.cuda.synchronize()
            t1 = time.time()
            if l == 0:
                # the index-build GEMM alone (exact KNN with the fused selection), HIP events on the launch stream
                ra.ra_knn(w.K, w.Q_prefill, w.knn)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                ra.ra_knn(w.K, w.Q_prefill, w.knn)
                e1.record()
                e1.synchronize()
                knn_ms = e0.elapsed_time(e1)
                knn_flop = 2.0 * w.Q_prefill.shape[0] * w.Q_prefill.shape[1] * w.Q_prefill.shape[2] * w.K.shape[2] * w.d
                knn_peak = MFMA_BF16_PEAK_TFLOPS if w.K.element_size() == 2 else MFMA_F32_PEAK_TFLOPS
                knn_rec = {"bound": "mfma", "ms_layer0": knn_ms, "achieved": knn_flop / (knn_ms * 1e-3) / 1e12,
                           "peak": knn_peak, "unit": "TFLOP/s", "frac": knn_flop / (knn_ms * 1e-3) / 1e12 / knn_peak}
                torch.cuda.synchronize()
                t1 = time.time()
            idx = ra.ra_build_index(w.K, w.Q_prefill, w.deg, w.knn)
            if not a.helpers:
                idx.configure(B.RA_CFG_HELPERS, B.RA_HELPERS_OFF)
            idx.configure(B.RA_CFG_SEEDS, seeds)
            if a.seed_shares is not None:
                idx.configure(B.RA_CFG_SEED_SHARES, a.seed_shares)
            k8 = ra.ra_quantize_keys(w.K) if a.q8 else None
            torch.cuda.synchronize()
            t2 = time.time()
            t_gen += t1 - t0
            t_build += t2 - t1
            n_q = w.Q_prefill.shape[1]
            M_prefill = w.Q_prefill.shape[2]
            build_flop += 2.0 * w.Q_prefill.shape[0] * n_q * w.Q_prefill.shape[2] * w.K.shape[2] * w.d
            layers.append(dict(K=w.K, V=w.V, q=w.q_decode, idx=idx, w=w, k8=k8))
            w.Q_prefill = None
            if l == 0 or (l + 1) % 8 == 0:
                log(f"{workload} layer {l + 1}/{nl}: generate {t1 - t0:.2f}s build {t2 - t1:.2f}s")
        w0 = layers[0]["w"]
        n_q, n_kv, d = layers[0]["q"].shape[2], w0.K.shape[1], w0.d
        T = layers[0]["q"].shape[0]
        topk, ef = topk or w0.topk, ef or w0.ef
        sink, window, deg_ = w0.sink, w0.window, w0.deg
        esz = w0.K.element_size()
        heads = n_seq * n_q
        for L in layers:
            L["out"] = torch.empty((n_seq, n_q, d), **f32)
            L["lse"] = torch.empty((n_seq, n_q), **f32)
            L["ids"] = torch.empty((n_seq, n_q, topk), dtype=torch.int32, device=dev)
            L["st"] = torch.zeros((n_seq, n_q, 4), dtype=torch.int32, device=dev)

        def one(L, t):
            ra.ra_decode_step(L["q"][t % T], L["idx"], L["K"], L["V"], sink, window, topk, ef, expand,
                              out=L["out"], lse=L["lse"], ids=L["ids"], stats=L["st"], k8=L["k8"])

        def step(t):
            for L in layers:
                one(L, t)

        # ---- timed region ---------------------------------------------------------------
        if a.graph:
            # one captured graph per distinct token index; workspaces are grown by an eager step first
            step(0)
            torch.cuda.synchronize()
            graphs = []
            cs = torch.cuda.Stream()
            for t in range(T):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.stream(cs):
                    with torch.cuda.graph(g, stream=cs):
                        step(t)
                graphs.append(g)
            torch.cuda.synchronize()
            run = lambda t: graphs[t % T].replay()
        else:
            run = step
        for t in range(warmup):
            run(t)
        torch.cuda.synchronize()
        # HIP events on the launch stream bracket the same timed region: the step is nothing but one fused
        # launch per layer, so their distance over (steps x layers) bounds that kernel's average launch time
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record()
        for t in range(steps):
            run(t)
        ev1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms_per_step = 1e3 * wall / steps
        decode_ms_region = ev0.elapsed_time(ev1) / (steps * len(layers))
        helpers_still_on = all(L["idx"].helpers_active for L in layers) if a.helpers else False
        seed_shares_on = all(L["idx"].seed_shares_active for L in layers) if a.helpers else False

        # spread of the step latency (a separate pass: one event pair per step, each step waited for)
        lat = []
        for t in range(max(steps, 20)):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            run(t)
            e1.record()
            e1.synchronize()
            lat.append(e0.elapsed_time(e1))
        lat.sort()
        p10_50_90 = [lat[int(0.1 * (len(lat) - 1))], lat[len(lat) // 2], lat[int(0.9 * (len(lat) - 1))]]

        def timed_train(fn, reps):
            # one event pair around a train of back-to-back launches captured in one graph: no host in
            # the loop, the gaps are the device's own (--graph 0: the same train launched eagerly)
            if not a.graph:
                for L in layers:
                    fn(L, 0)
                torch.cuda.synchronize()
                s_, e_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                s_.record()
                for r in range(reps):
                    for L in layers:
                        fn(L, r)
                e_.record()
                torch.cuda.synchronize()
                return s_.elapsed_time(e_) / (reps * len(layers))
            g = torch.cuda.CUDAGraph()
            cs2 = torch.cuda.Stream()
            with torch.cuda.stream(cs2):
                with torch.cuda.graph(g, stream=cs2):
                    for r in range(reps):
                        for L in layers:
                            fn(L, r)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            s_, e_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s_.record()
            g.replay()
            e_.record()
            torch.cuda.synchronize()
            return s_.elapsed_time(e_) / (reps * len(layers))

        # Both live figures bound the kernel's duration from above: events around the timed region also
        # see the start-up of every graph replay (it matters when a step is a single launch); a train of
        # launches in one graph leaves only the gaps between launches. The smaller one is reported; it is
        # the one the rocprofv3 kernel trace agrees with.
        reps = max(4, 64 // len(layers))
        decode_ms_train = timed_train(one, reps)
        decode_ms = min(decode_ms_region, decode_ms_train)
        stats_sum = np.zeros(4, np.float64)
        for t in range(T):
            step(t)
            torch.cuda.synchronize()
            for L in layers:
                stats_sum += L["st"].double().sum(dim=(0, 1)).cpu().numpy()
        n_launch = T * len(layers)
        visited, expanded, iters, returned = stats_sum / n_launch      # per launch (all heads)
        # algorithmic bytes of one launch: key rows scored + adjacency rows read + q + ids (search),
        # retrieved K/V rows per query head + static K/V rows per KV head (attention)
        key_row_bytes = d * (1 if a.q8 else esz)           # what the walk reads per scored key
        search_bytes = visited * key_row_bytes + expanded * deg_ * 4 + heads * (d * esz + topk * 4)
        W = min(N, sink + window)
        attend_bytes = returned * 2 * d * esz + n_seq * n_kv * W * 2 * d * esz
        decode_bytes = search_bytes + attend_bytes
        decode_gbs = decode_bytes / (decode_ms * 1e-3) / 1e9

        # recall of the graph search against the exact scan, every head of every layer, on the device
        flat_ws = torch.empty(ra.lib().ra_flat_workspace_bytes(n_seq, n_q, N), dtype=torch.uint8, device=dev)
        flat_ids = torch.empty((n_seq, n_q, topk), dtype=torch.int32, device=dev)
        t_last = (steps - 1) % T
        hits = total = 0
        for L in layers:
            one(L, t_last)
            ra.ra_flat_topk(L["q"][t_last], L["K"], sink, window, topk, workspace=flat_ws, ids=flat_ids)
            got, ref = L["ids"].long(), flat_ids.long()
            match = (got.unsqueeze(-1) == ref.unsqueeze(-2)) & (ref.unsqueeze(-2) >= 0)
            hits += int(match.any(-2).sum())
            total += int((ref >= 0).sum())
        recall_device = hits / max(total, 1)

        res = {
            "ms_per_step": ms_per_step, "step_ms_p10_p50_p90": p10_50_90,
            "recall_at_k": recall_device,
            "config": {"workload": f"{workload}: {len(layers)} layers x {n_seq} seq x {n_q} q heads / "
                                   f"{n_kv} kv heads, d={d}, N={N}, M={M_prefill} prefill queries/head",
                       "topk": topk, "ef": ef, "expand": expand, "seeds": seeds, "deg": deg_, "knn": w0.knn,
                       "sink": sink, "window": window, "hip_graph": bool(a.graph),
                       "search_keys": "int8" if a.q8 else "as stored"},
            "roofline": {"bound": "hbm", "kernel": "decode_kernel", "achieved": decode_gbs,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": decode_gbs / HBM_PEAK_GBS,
                         "traffic": None if (a.q8 or context or not a.helpers) else
                         traffic_from_profiles(workload, seeds, ef, expand),
                         "avg_launch_ms": decode_ms, "avg_launch_ms_timed_region": decode_ms_region,
                         "avg_launch_ms_graph_train": decode_ms_train,
                         "algorithmic_bytes_per_launch": decode_bytes,
                         "visited_per_search": visited / heads, "expanded_per_search": expanded / heads,
                         "iters_per_search": iters / heads,
                         "helper_workgroups_active_after_timed_region": helpers_still_on,
                         "seed_workgroups_active_after_timed_region": seed_shares_on},
            "build": {"seconds": t_build, "generate_seconds": t_gen,
                      "knn_TFLOPs_incl_projection": build_flop / max(t_build, 1e-9) / 1e12, "knn_kernel": knn_rec},
        }
        state = dict(layers=layers, one=one, step=step, timed_train=timed_train, T=T, N=N, n_seq=n_seq, n_q=n_q,
                     n_kv=n_kv, d=d, esz=esz, topk=topk, ef=ef, sink=sink, window=window, deg=deg_, expand=expand,
                     seeds=seeds, heads=heads, flat_ws=flat_ws, flat_ids=flat_ids, t_last=t_last,
                     search_bytes=search_bytes, attend_bytes=attend_bytes, decode_ms=decode_ms)
        return res, state

    res, S = measure(a.workload, a.steps, a.warmup, a.tokens, n_layers=a.layers, context=a.context, seqs=a.seqs,
                     topk=a.topk, ef=a.ef, deg=a.deg, knn=a.knn, expand=a.expand, seeds=a.seeds)
    layers, T, N, n_seq, n_q, n_kv, d, esz = (S[k] for k in ("layers", "T", "N", "n_seq", "n_q", "n_kv", "d", "esz"))
    topk, ef, sink, window, expand, seeds, heads = (S[k] for k in ("topk", "ef", "sink", "window", "expand", "seeds",
                                                                   "heads"))

    # ---- the stand-alone stage kernels, timed the same way, for the breakdown ---------------------
    dt_code = 1 if esz == 2 else 0
    L_ = ra.lib()

    def search_only(L, t):
        rc = L_.ra_search(L["q"][t % T].data_ptr(), L["idx"].handle, L["K"].data_ptr(), dt_code, N,
                          sink, window, topk, ef, expand,
                          torch.cuda.current_stream().cuda_stream, L["ids"].data_ptr(),
                          L["st"].data_ptr())
        assert rc == 0, L_.ra_last_error()

    def attend_only(L, t):
        rc = L_.ra_attend(L["q"][t % T].data_ptr(), L["idx"].handle, L["K"].data_ptr(),
                          L["V"].data_ptr(), dt_code, N, sink, window, topk, L["ids"].data_ptr(),
                          torch.cuda.current_stream().cuda_stream, L["out"].data_ptr(),
                          L["lse"].data_ptr(), None, None, None, None)
        assert rc == 0, L_.ra_last_error()

    for L in layers:                            # every handle's workspace grows before a capture
        search_only(L, 0)
        attend_only(L, 0)
    torch.cuda.synchronize()
    reps = max(4, 64 // len(layers))
    search_ms = S["timed_train"](search_only, reps)
    attend_ms = S["timed_train"](attend_only, reps)

    # ---- exact baselines on the same data (the paper's "Flat" retrieval and full attention) ---
    full_ws = torch.empty(ra.lib().ra_full_attention_workspace_bytes(n_seq, n_q, n_kv, N),
                          dtype=torch.uint8, device=dev)
    f_out, f_lse = torch.empty((n_seq, n_q, d), **f32), torch.empty((n_seq, n_q), **f32)
    base_layers = layers[:min(len(layers), 4)]

    def timed_layers(fn, reps=5):
        """ms per layer of an exact baseline, replayed from a HIP graph like the decode step (eager
        launches with --graph 0), so that the comparison is between kernels, not launch paths."""
        fn(base_layers[0])
        torch.cuda.synchronize()
        graph = None
        if a.graph:
            cs = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(cs):
                with torch.cuda.graph(graph, stream=cs):
                    for L in base_layers:
                        fn(L)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            if graph is not None:
                graph.replay()
            else:
                for L in base_layers:
                    fn(L)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (reps * len(base_layers))

    t_last = S["t_last"]
    flat_ms = timed_layers(lambda L: ra.ra_flat_topk(L["q"][t_last], L["K"], sink, window, topk,
                                                     workspace=S["flat_ws"], ids=S["flat_ids"]))
    full_ms = timed_layers(lambda L: ra.ra_full_attention(L["q"][t_last], L["K"], L["V"],
                                                          workspace=full_ws, out=f_out, lse=f_lse))
    key_bytes = n_seq * n_kv * N * d * esz
    del full_ws

    # ---- what the device's memory sustains: a plain 1 GiB copy and a read-only streaming kernel -----
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    fold = torch.zeros(1, dtype=torch.int64, device=dev)

    def gbs(fn, nbytes, reps=5):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9

    copy_gbs = gbs(lambda: dst.copy_(src), 2.0 * (1 << 30))
    read_gbs = gbs(lambda: ra.ra_hbm_read_probe(src, fold), 1.0 * (1 << 30))
    # scattered rows of 256 B (a bf16 key), as many bytes as the buffer holds, 16 lanes per row
    gather_gbs = gbs(lambda: ra.ra_hbm_gather_probe(src, (1 << 30) // 256, fold), 1.0 * (1 << 30))
    if a.copy_calibration:
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    del src, dst
    hbm_measured = {"copy_1GiB_read_plus_write_GBs": copy_gbs, "read_stream_1GiB_GBs": read_gbs,
                    "gather_256B_rows_of_1GiB_GBs": gather_gbs,
                    "peak_GBs": HBM_PEAK_GBS,
                    "decode_kernel_frac_of_read_stream": res["roofline"]["achieved"] / read_gbs,
                    "decode_kernel_frac_of_gather": res["roofline"]["achieved"] / gather_gbs}

    # ---- recall@k against brute force (CPU oracle) on a sample of layers ---------------
    from oracle import attention as OA, mips as OM
    rec = []
    Wset = OA.static_ids(N, sink, window)
    rl = list(range(0, len(layers), max(1, len(layers) // max(1, a.recall_layers))))[:a.recall_layers]
    for li in rl:
        L = layers[li]
        S["one"](L, t_last)
        ids = L["ids"].cpu().numpy()
        for s in range(n_seq):
            for kvh in range(n_kv):
                Kh = L["K"][s, kvh].float().cpu().numpy()
                for j in range(n_q // n_kv):
                    h = kvh * (n_q // n_kv) + j
                    qv = L["q"][t_last, s, h].float().cpu().numpy()
                    truth = OM.topk_bruteforce(qv, Kh, topk, exclude=Wset)
                    rec.append(OM.recall(ids[s, h], truth))
    recall = float(np.mean(rec)) if rec else None

    # ---- the other BASELINE configurations, measured the same way ----------------------------------
    other = None
    if a.workload == "config2" and not a.no_other_configs and not (a.layers or a.context or a.q8):
        other = {}
        for wl, st_, tk in (("config3", 20, 4), ("config4", 10, 4)):
            r, s2 = measure(wl, st_, 2, tk)
            r["ms_per_launch"] = r["roofline"]["avg_launch_ms"]
            r["roofline"]["frac_of_measured_gather"] = r["roofline"]["achieved"] / gather_gbs
            other[wl] = r
            for L in s2["layers"]:
                L["idx"].free()
            del s2
            torch.cuda.empty_cache()

    # ---- CPU baseline: the oracle's decode step on a bounded sample of heads, over the host's cores --
    cpu = None
    if not a.no_cpu_baseline and not a.q8:
        L = layers[0]
        S["one"](L, t_last)
        ids_gpu = L["ids"].cpu().numpy()
        n_cpu = min(a.cpu_heads, n_q)
        n_tok = min(a.cpu_tokens, T)
        tokens = [(t_last + i) % T for i in range(n_tok)]      # starts with the token the GPU ids are from
        ref, wall, work, workers = cpu_baseline(ra, L, n_q, n_kv, tokens, a.cpu_workers, sink, window, topk, ef,
                                                expand, seeds, list(range(n_cpu)), len(layers))
        same = sum(int(ref[h].tolist() == ids_gpu[0, h].tolist()) for h in ref)
        per_head_wall_ms = 1e3 * wall / (n_cpu * n_tok)
        cpu = {"value": per_head_wall_ms * heads * len(layers), "unit": "ms", "cores": workers, "kind": "oracle",
               "sample": f"{n_cpu} query heads of layer 0 x {n_tok} decode queries at the full context, one head per "
                         f"host process over {workers} processes ({wall:.1f} s of wall clock, {work:.1f} s of CPU "
                         f"work), scaled to one token = {heads} heads x {len(layers)} layers; {same}/{len(ref)} "
                         f"heads returned ids identical to the GPU",
               "single_core_ms": 1e3 * work / (n_cpu * n_tok) * heads * len(layers)}

    out = {
        "metric": METRIC,
        "value": res["ms_per_step"], "unit": "ms", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": res["ms_per_step"], "step_ms_p10_p50_p90": res["step_ms_p10_p50_p90"],
        "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if esz == 2 else "f32", "data": "synthetic",
        "recall_at_100": res["recall_at_k"], "recall_at_100_cpu_oracle_sample": recall,
        "config": res["config"],
        "roofline": res["roofline"],
        "hbm_measured": hbm_measured,
        "stages": {"ra_search": {"avg_launch_ms": search_ms,
                                 "algorithmic_GBs": S["search_bytes"] / (search_ms * 1e-3) / 1e9,
                                 "algorithmic_bytes_per_launch": S["search_bytes"]},
                   "ra_attend": {"avg_launch_ms": attend_ms,
                                 "algorithmic_GBs": S["attend_bytes"] / (attend_ms * 1e-3) / 1e9,
                                 "algorithmic_bytes_per_launch": S["attend_bytes"]}},
        "exact_baselines": {
            "flat_topk": {"ms_per_layer": flat_ms, "key_scan_GBs": key_bytes / (flat_ms * 1e-3) / 1e9,
                          "frac_of_hbm_peak": key_bytes / (flat_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                          "frac_of_read_stream": key_bytes / (flat_ms * 1e-3) / 1e9 / read_gbs},
            "full_attention": {"ms_per_layer": full_ms,
                               "kv_scan_GBs": 2 * key_bytes / (full_ms * 1e-3) / 1e9,
                               "frac_of_hbm_peak": 2 * key_bytes / (full_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                               "frac_of_read_stream": 2 * key_bytes / (full_ms * 1e-3) / 1e9 / read_gbs},
            "graph_decode_ms_per_layer": S["decode_ms"]},
        "build": res["build"],
        "other_configs": other,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
