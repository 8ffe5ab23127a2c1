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
HBM traffic the counters read), `stages`, `exact_baselines`, `build` (with `knn_kernel`: the
index-build GEMM's live time for one layer against the dense MFMA peak), `cpu_baseline`.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes per decode_kernel launch of the default workload, from the two rocprofv3 --pmc runs
# summarised under profiles/ (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, KiB per dispatch, scale factors
# from a 1 GiB device copy in the same runs).
DECODE_TRAFFIC_BYTES_CONFIG2 = 13988278
MFMA_BF16_PEAK_TFLOPS = 2500.0
MFMA_F32_PEAK_TFLOPS = 157.3


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
    p.add_argument("--expand", type=int, default=None,
                   help="search expansion width (default 64; 16 for config4; 32 for config3, where the smaller "
                        "candidate buffers let more searches share a compute unit)")
    p.add_argument("--tokens", type=int, default=8, help="distinct decode queries per head")
    p.add_argument("--recall-layers", type=int, default=2)
    p.add_argument("--cpu-heads", type=int, default=32, help="heads the CPU oracle is timed on")
    p.add_argument("--cpu-tokens", type=int, default=8, help="decode queries per head the CPU oracle is timed on")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--graph", type=int, default=1, help="replay the step from a captured HIP graph")
    p.add_argument("--q8", type=int, default=0,
                   help="1: the graph walk reads an 8-bit copy of the keys (ra_decode_step_q8)")
    p.add_argument("--helpers", type=int, default=1,
                   help="0: every head attends to the static set itself (no helper workgroups)")
    p.add_argument("--copy-calibration", action="store_true",
                   help="also run three plain 1 GiB device copies (reference for HBM counters)")
    return p.parse_args()


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards without exchange over "
              "layers, heads and sequences). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2409_10516_amd as ra
    from paper_2409_10516_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if a.expand is None:
        a.expand = {"config3": 32, "config4": 16}.get(a.workload, 64)
    if a.q8 and not a.no_cpu_baseline:
        print("bench.py: --q8 runs skip the CPU baseline (it times the oracle's walk over the keys as stored)",
              file=sys.stderr)
        a.no_cpu_baseline = True
    dev = "cuda:0"
    torch.cuda.set_device(0)
    ra.lib()                                    # fail loudly if the HIP library is missing

    # ---- workload -------------------------------------------------------------------
    if a.workload == "config2":
        n_layers, N, n_seq = 32, 131072, 1
        kw = {k: v for k, v in (('deg', a.deg), ('knn', a.knn)) if v}
        mk = lambda l: synth.make_config2_layer(l, device=dev, N=N, T=a.tokens, **kw)
    elif a.workload == "config1":
        n_layers, N, n_seq = 1, 32768, 1
        mk = lambda l: synth.make_config1(device=dev, N=N, T=a.tokens)
    elif a.workload == "config3":
        n_layers, N, n_seq = 1, 32768, a.seqs or 16
        mk = lambda l: synth.make_config3(device=dev, N=N, T=a.tokens, n_seq=n_seq)
    elif a.workload == "config4":
        n_layers, N, n_seq = 1, 1 << 20, 1
        mk = lambda l: synth.make_config4(device=dev, N=N, T=a.tokens)
    else:
        n_layers, N, n_seq = 1, 4096, 1
        mk = lambda l: synth.make_config0(device=dev)
    if a.context:
        N = a.context
    if a.layers:
        n_layers = a.layers

    layers = []
    t_gen = t_build = 0.0
    build_flop = 0.0
    for l in range(n_layers):
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
            torch.cuda.synchronize()
            t1 = time.time()
        idx = ra.ra_build_index(w.K, w.Q_prefill, w.deg, w.knn)
        if not a.helpers:
            idx.configure(ra.binding.RA_CFG_HELPERS, ra.binding.RA_HELPERS_OFF)
        k8 = ra.ra_quantize_keys(w.K) if a.q8 else None
        torch.cuda.synchronize()
        t2 = time.time()
        t_gen += t1 - t0
        t_build += t2 - t1
        n_q = w.Q_prefill.shape[1]
        m_prefill = w.Q_prefill.shape[2]
        build_flop += 2.0 * w.Q_prefill.shape[0] * n_q * w.Q_prefill.shape[2] * w.K.shape[2] * w.d
        layers.append(dict(K=w.K, V=w.V, q=w.q_decode, idx=idx, w=w, k8=k8))
        w.Q_prefill = None
        if l == 0 or (l + 1) % 8 == 0:
            print(f"[bench] layer {l + 1}/{n_layers}: generate {t1 - t0:.2f}s build {t2 - t1:.2f}s",
                  file=sys.stderr, flush=True)
    w0 = layers[0]["w"]
    n_q, n_kv, d = layers[0]["q"].shape[2], w0.K.shape[1], w0.d
    M_prefill = m_prefill
    T = layers[0]["q"].shape[0]
    topk, ef, sink, window, deg = a.topk or w0.topk, a.ef or w0.ef, w0.sink, w0.window, w0.deg
    esz = w0.K.element_size()
    heads = n_seq * n_q
    f32 = dict(dtype=torch.float32, device=dev)
    for L in layers:
        L["out"] = torch.empty((n_seq, n_q, d), **f32)
        L["lse"] = torch.empty((n_seq, n_q), **f32)
        L["ids"] = torch.empty((n_seq, n_q, topk), dtype=torch.int32, device=dev)
        L["st"] = torch.zeros((n_seq, n_q, 4), dtype=torch.int32, device=dev)

    def step(t):
        for L in layers:
            ra.ra_decode_step(L["q"][t % T], L["idx"], L["K"], L["V"], sink, window, topk, ef,
                              a.expand, out=L["out"], lse=L["lse"], ids=L["ids"], stats=L["st"], k8=L["k8"])

    dt_code = 1 if esz == 2 else 0
    L_ = ra.lib()

    def search_only(L, t):
        rc = L_.ra_search(L["q"][t % T].data_ptr(), L["idx"].handle, L["K"].data_ptr(), dt_code, N,
                          sink, window, topk, ef, a.expand,
                          torch.cuda.current_stream().cuda_stream, L["ids"].data_ptr(),
                          L["st"].data_ptr())
        assert rc == 0, L_.ra_last_error()

    def attend_only(L, t):
        rc = L_.ra_attend(L["q"][t % T].data_ptr(), L["idx"].handle, L["K"].data_ptr(),
                          L["V"].data_ptr(), dt_code, N, sink, window, topk, L["ids"].data_ptr(),
                          torch.cuda.current_stream().cuda_stream, L["out"].data_ptr(),
                          L["lse"].data_ptr(), None, None, None, None)
        assert rc == 0, L_.ra_last_error()

    # ---- timed region ---------------------------------------------------------------
    graphs = None
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
    for t in range(a.warmup):
        run(t)
    torch.cuda.synchronize()
    # HIP events on the launch stream bracket the same timed region: the step is nothing but one fused
    # launch per layer, so their distance over (steps x layers) is that kernel's average launch time
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for t in range(a.steps):
        run(t)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = 1e3 * wall / a.steps
    decode_ms_region = ev0.elapsed_time(ev1) / (a.steps * len(layers))

    # spread of the step latency (a separate pass: one event pair per step, each step waited for)
    lat = []
    for t in range(max(a.steps, 20)):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run(t)
        e1.record()
        e1.synchronize()
        lat.append(e0.elapsed_time(e1))
    lat.sort()
    step_ms_p10_p50_p90 = [lat[int(0.1 * (len(lat) - 1))], lat[len(lat) // 2], lat[int(0.9 * (len(lat) - 1))]]

    # ---- dominant kernel: live HIP-event timing on the launch stream ----------------------
    # The timed region launches one fused kernel per layer (decode_kernel: search, sparse and
    # static attention, combination). Besides the events around the timed region it is timed here
    # launch by launch; the stand-alone stage kernels (ra_search, ra_attend) are timed the same way
    # for the breakdown.
    def timed_pass(fn):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(a.steps * len(layers))]
        i = 0
        for t in range(a.steps):
            for L in layers:
                evs[i][0].record()
                fn(L, t)
                evs[i][1].record()
                i += 1
        torch.cuda.synchronize()
        return sum(s_.elapsed_time(e_) for s_, e_ in evs) / len(evs)

    def timed_train(fn):
        # one event pair around a train of back-to-back launches: the host enqueues faster than
        # the device runs them, so the stream never drains and the gaps are the device's own
        for L in layers:
            fn(L, 0)
        torch.cuda.synchronize()
        s_, e_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s_.record()
        for t in range(a.steps):
            for L in layers:
                fn(L, t)
        e_.record()
        torch.cuda.synchronize()
        return s_.elapsed_time(e_) / (a.steps * len(layers))

    def fused_only(L, t):
        ra.ra_decode_step(L["q"][t % T], L["idx"], L["K"], L["V"], sink, window, topk, ef, a.expand,
                          out=L["out"], lse=L["lse"], ids=L["ids"], stats=L["st"], k8=L["k8"])

    stats_sum = np.zeros(4, np.float64)
    # All live figures bound the kernel's duration from above: events around the timed region
    # also see the start-up of every graph replay (it matters when a step is a single launch),
    # events around each eager launch the gap between an event and the launch behind it (it
    # matters when a launch is short), events around a train of eager launches the gaps between
    # launches. The smallest one is the kernel's; it is the one the rocprofv3 kernel trace agrees with.
    decode_ms_eager = timed_pass(fused_only)
    decode_ms_train = timed_train(fused_only)
    decode_ms = min(decode_ms_region, decode_ms_eager, decode_ms_train)
    for t in range(T):
        step(t)
        torch.cuda.synchronize()
        for L in layers:
            stats_sum += L["st"].double().sum(dim=(0, 1)).cpu().numpy()
    search_ms = timed_pass(search_only)
    attend_ms = timed_pass(attend_only)
    n_launch = T * len(layers)
    visited, expanded, iters, returned = stats_sum / n_launch      # per launch (all heads)
    # algorithmic bytes of one launch: key rows scored + adjacency rows read + q + ids (search),
    # retrieved K/V rows per query head + static K/V rows per KV head (attention)
    key_row_bytes = d * (1 if a.q8 else esz)           # what the walk reads per scored key
    search_bytes = visited * key_row_bytes + expanded * deg * 4 + heads * (d * esz + topk * 4)
    W = min(N, sink + window)
    attend_bytes = returned * 2 * d * esz + n_seq * n_kv * W * 2 * d * esz
    decode_bytes = search_bytes + attend_bytes
    decode_gbs = decode_bytes / (decode_ms * 1e-3) / 1e9
    search_gbs = search_bytes / (search_ms * 1e-3) / 1e9
    attend_gbs = attend_bytes / (attend_ms * 1e-3) / 1e9

    # ---- exact baselines on the same data (the paper's "Flat" retrieval and full attention) ---
    flat_ws = torch.empty(ra.lib().ra_flat_workspace_bytes(n_seq, n_q, N), dtype=torch.uint8, device=dev)
    full_ws = torch.empty(ra.lib().ra_full_attention_workspace_bytes(n_seq, n_q, n_kv, N),
                          dtype=torch.uint8, device=dev)
    flat_ids = torch.empty((n_seq, n_q, topk), dtype=torch.int32, device=dev)
    f_out, f_lse = torch.empty((n_seq, n_q, d), **f32), torch.empty((n_seq, n_q), **f32)
    base_layers = layers[:min(len(layers), 4)]

    def timed_layers(fn, reps=5):
        fn(base_layers[0])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            for L in base_layers:
                fn(L)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (reps * len(base_layers))

    t_last = (a.steps - 1) % T
    flat_ms = timed_layers(lambda L: ra.ra_flat_topk(L["q"][t_last], L["K"], sink, window, topk,
                                                     workspace=flat_ws, ids=flat_ids))
    full_ms = timed_layers(lambda L: ra.ra_full_attention(L["q"][t_last], L["K"], L["V"],
                                                          workspace=full_ws, out=f_out, lse=f_lse))
    key_bytes = n_seq * n_kv * N * d * esz
    # recall of the graph search against the exact scan, every head of every layer, on the device
    hits = total = 0
    for L in layers:
        ra.ra_decode_step(L["q"][t_last], L["idx"], L["K"], L["V"], sink, window, topk, ef, a.expand,
                          out=L["out"], lse=L["lse"], ids=L["ids"], stats=L["st"], k8=L["k8"])
        ra.ra_flat_topk(L["q"][t_last], L["K"], sink, window, topk, workspace=flat_ws, ids=flat_ids)
        got, ref = L["ids"].long(), flat_ids.long()
        match = (got.unsqueeze(-1) == ref.unsqueeze(-2)) & (ref.unsqueeze(-2) >= 0)
        hits += int(match.any(-2).sum())
        total += int((ref >= 0).sum())
    recall_device = hits / max(total, 1)
    del flat_ws, full_ws

    if a.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- recall@100 against brute force (CPU oracle) on a sample of layers ---------------
    from oracle import attention as OA, mips as OM
    rec = []
    Wset = OA.static_ids(N, sink, window)
    rl = list(range(0, len(layers), max(1, len(layers) // max(1, a.recall_layers))))[:a.recall_layers]
    for li in rl:
        L = layers[li]
        ids = L["ids"].cpu().numpy()                 # from the last timed token
        t_last = (a.steps - 1) % T
        for s in range(n_seq):
            for kvh in range(n_kv):
                Kh = L["K"][s, kvh].float().cpu().numpy()
                for j in range(n_q // n_kv):
                    h = kvh * (n_q // n_kv) + j
                    qv = L["q"][t_last, s, h].float().cpu().numpy()
                    truth = OM.topk_bruteforce(qv, Kh, topk, exclude=Wset)
                    rec.append(OM.recall(ids[s, h], truth))
    recall = float(np.mean(rec)) if rec else None

    # ---- CPU baseline: the oracle's decode step on a bounded sample of heads --------------
    cpu = None
    if not a.no_cpu_baseline:
        from oracle import decode as OD
        L = layers[0]
        n_cpu = min(a.cpu_heads, n_q)
        t_last = (a.steps - 1) % T
        ids_gpu = L["ids"].cpu().numpy()
        prepared = []
        for h in range(n_cpu):
            adj, ent = ra.ra_index_export(L["idx"], 0, h)
            kvh = h // (n_q // n_kv)
            prepared.append((h, L["K"][0, kvh].float().cpu().numpy(),
                             L["V"][0, kvh].float().cpu().numpy(), adj.numpy(), ent))
        n_tok = min(a.cpu_tokens, T)
        qs = L["q"].float().cpu().numpy()
        tc = time.perf_counter()
        ref_last = {}
        for t in [(t_last + i) % T for i in range(n_tok)]:      # starts with the token the GPU ids are from
            for h, Kh, Vh, adj, ent in prepared:
                _, _, r_ids, _ = OD.decode_step(qs[t, 0, h], Kh, Vh, adj, ent, sink, window, topk, ef,
                                                a.expand)
                if t == t_last:
                    ref_last[h] = r_ids
        cpu_s = time.perf_counter() - tc
        same = sum(int(ref_last[h].tolist() == ids_gpu[0, h].tolist()) for h in ref_last)
        per_head_ms = 1e3 * cpu_s / (n_cpu * n_tok)
        cpu = {"value": per_head_ms * heads * len(layers), "unit": "ms", "cores": 1,
               "kind": "oracle",
               "sample": f"{n_cpu} query heads of layer 0 x {n_tok} decode queries at the full context "
                         f"({cpu_s:.1f} s of CPU work, one thread), scaled to one token = {heads} heads x "
                         f"{len(layers)} layers; {same}/{len(ref_last)} heads returned ids identical to "
                         f"the GPU"}

    out = {
        "metric": "decode-step retrieval-attention latency (ms) @128K ctx, 1 GPU; recall@100",
        "value": ms_per_step, "unit": "ms", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "step_ms_p10_p50_p90": step_ms_p10_p50_p90, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if esz == 2 else "f32", "data": "synthetic",
        "recall_at_100": recall_device, "recall_at_100_cpu_oracle_sample": recall,
        "config": {"workload": f"{a.workload}: {len(layers)} layers x {n_seq} seq x {n_q} q heads / "
                               f"{n_kv} kv heads, d={d}, N={N}, M={M_prefill} prefill queries/head",
                   "topk": topk, "ef": ef, "expand": a.expand, "deg": deg, "knn": w0.knn,
                   "sink": sink, "window": window, "hip_graph": bool(a.graph), "search_keys": "int8" if a.q8 else "as stored"},
        "roofline": {"bound": "hbm", "kernel": "decode_kernel", "achieved": decode_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": decode_gbs / HBM_PEAK_GBS,
                     "traffic": (DECODE_TRAFFIC_BYTES_CONFIG2 if (a.workload == "config2"
                                 and a.expand == 64 and not a.context) else None),
                     "avg_launch_ms": decode_ms, "avg_launch_ms_timed_region": decode_ms_region,
                     "avg_launch_ms_eager_events": decode_ms_eager,
                     "avg_launch_ms_eager_train": decode_ms_train,
                     "algorithmic_bytes_per_launch": decode_bytes,
                     "visited_per_search": visited / heads, "expanded_per_search": expanded / heads,
                     "iters_per_search": iters / heads},
        "stages": {"ra_search": {"avg_launch_ms": search_ms, "algorithmic_GBs": search_gbs,
                                 "algorithmic_bytes_per_launch": search_bytes},
                   "ra_attend": {"avg_launch_ms": attend_ms, "algorithmic_GBs": attend_gbs,
                                 "algorithmic_bytes_per_launch": attend_bytes}},
        "exact_baselines": {
            "flat_topk": {"ms_per_layer": flat_ms, "key_scan_GBs": key_bytes / (flat_ms * 1e-3) / 1e9,
                          "frac_of_hbm_peak": key_bytes / (flat_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "full_attention": {"ms_per_layer": full_ms,
                               "kv_scan_GBs": 2 * key_bytes / (full_ms * 1e-3) / 1e9,
                               "frac_of_hbm_peak": 2 * key_bytes / (full_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "graph_decode_ms_per_layer": decode_ms},
        "build": {"seconds": t_build, "generate_seconds": t_gen,
                  "knn_TFLOPs_incl_projection": build_flop / max(t_build, 1e-9) / 1e12,
                  "knn_kernel": {"bound": "mfma", "ms_layer0": knn_ms, "achieved": knn_flop / (knn_ms * 1e-3) / 1e12,
                                 "peak": knn_peak, "unit": "TFLOP/s",
                                 "frac": knn_flop / (knn_ms * 1e-3) / 1e12 / knn_peak}},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
