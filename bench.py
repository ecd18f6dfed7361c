#!/usr/bin/env python3
"""Benchmark of the IceCache hot path on one MI355X.

Workload (default): the Llama-3-8B-shaped layer of the benchmark definition -- batch 1, 8 KV heads /
32 query heads, head_dim 128, context 32768, page_size 16, 512 clusters per KV head, token budget
256 -- for 32 independently seeded layers.  One "step" is one decode token's select+attend over all
32 layers (256 units).  Printed value: microseconds per layer-step with the 32 independent layers
batched in one launch set; the one-layer-at-a-time figure (HIP-graph replay of 32 dependent-order
launches) is reported beside it, together with the index build (clustering) and insertion timings,
the roofline of the dominant kernel and the CPU oracle timed on the host cores.

All inputs are seeded synthetic data (datagen.py) resident in HBM before the timed region.  No timed
step may find its index in L2 or in the 256 MB memory-side cache: the headline loop rotates over
three copies of the index (540 MB of lines per round) with one event pair around all steps; the
per-step figures (percentiles, select-only, attend-only, one-layer-at-a-time) bracket every step
with its own event pair and READ a 1 GiB buffer (untimed) before it.  (Reading rather than writing
the buffer leaves clean lines behind; dirty lines would add write-back traffic to the timed
kernel.)  Every figure labelled "cold" is therefore an HBM figure.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import datagen  # noqa: E402

HBM_PEAK_GBPS = 8000.0
# HBM bytes of one batched decode_step launch (fetch + write), from the counter runs summarised in
# profiles/decode_step_cfg2_hbm_counters.md; refreshed whenever that profile is.
MEASURED_TRAFFIC_BYTES = 180154 * 1024
MFMA_BF16_PEAK_TFLOPS = 2500.0
D = 128


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layers", type=int, default=0,
                    help="independent (layer or sequence) index sets batched in one launch; default 32 / 1 / 16 for cfg2 / 3 / 4")
    ap.add_argument("--kmeans-iters", type=int, default=10)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg3", "cfg4"],
                    help="cfg2 is the headline; cfg3 (131k context, budget 1024) and cfg4 (16 sequences) are extra shapes")
    ap.add_argument("--n-probe", type=int, default=0, help="clusters kept by the hierarchical variant (default n_clusters / 8)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--warm", action="store_true", help="skip the cache flush between steps")
    return ap.parse_args()


def gen_layer(w, layer):
    K, V = datagen.keys_values(w, seed=w.seed + layer)
    return K[0], V[0], datagen.init_indices(w, seed=w.seed + layer)[0], datagen.queries(w, seed=w.seed + layer)[0]


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every unit is independent; more GPUs would just "
              "take disjoint heads or sequences); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_10539_amd import IceIndex, ice_debug_peak_mfma, ice_debug_peak_read, ice_select, ice_select_attend_resident, ice_select_hier

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    import dataclasses
    w = dataclasses.replace(datagen.WORKLOADS[args.workload], batch=1)   # sequences of cfg4 are generated like layers
    if args.layers <= 0:
        args.layers = {"cfg2": 32, "cfg3": 1, "cfg4": 16}[args.workload]
    if args.n_probe <= 0:
        args.n_probe = max(1, w.n_clusters // 8)
    L, H, G, n, s, C, budget = args.layers, w.n_kv_heads, w.group_size, w.n_tokens, w.page_size, w.n_clusters, w.token_budget
    P = budget // s
    T = args.kmeans_iters
    max_tokens = n + 128

    t0 = time.time()
    with ThreadPoolExecutor(max_workers=min(16, L)) as ex:
        layers = list(ex.map(lambda l: gen_layer(w, l), range(L)))
    K = torch.from_numpy(np.stack([x[0] for x in layers]).view(np.int16)).to(dev)       # [L,H,n,d]
    V = torch.from_numpy(np.stack([x[1] for x in layers]).view(np.int16)).to(dev)
    init = torch.from_numpy(np.stack([x[2] for x in layers])).to(dev)                   # [L,H,C]
    q_np = np.stack([x[3] for x in layers])                                             # [L,H*G,d]
    K0_np, init0_np = layers[0][0][0].copy(), layers[0][2][0].copy()                    # one unit, for the oracle
    q = torch.from_numpy(q_np.view(np.int16)).to(dev)
    del layers
    t_gen = time.time() - t0

    def ev():
        return torch.cuda.Event(enable_timing=True)

    st = torch.cuda.current_stream()

    # ---------------------------------------------------------------- index build (clustering + paging)
    # (a) one index per layer (B=1, 8 units): the one-layer-at-a-time decode path
    per_layer = [IceIndex(1, H, G, max_tokens, s, C, kmeans_iters=T, init_idx=init[l].contiguous(), device=dev)
                 for l in range(L)]
    per_layer[0].build_index(K[0], V[0])          # warm-up of every build kernel
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record(st)
    for l in range(L):
        per_layer[l].build_index(K[l], V[l])
    e1.record(st)
    torch.cuda.synchronize()
    build_ms_layer = e0.elapsed_time(e1) / L
    # (b) all layers as one batch of 256 units: the batched decode path
    batched = IceIndex(L, H, G, max_tokens, s, C, kmeans_iters=T, init_idx=init.contiguous(), device=dev)
    e0, e1 = ev(), ev()
    e0.record(st)
    batched.build_index(K, V)
    e1.record(st)
    torch.cuda.synchronize()
    build_ms_batched = e0.elapsed_time(e1)
    assign_flop_round = 2.0 * n * C * D * H * L

    def build_ms(layers_, T_, K_, V_, init_, geometry=0):
        ix = IceIndex(layers_, H, G, max_tokens, s, C, kmeans_iters=T_, init_idx=init_, device=dev, geometry=geometry)
        ix.build_index(K_, V_)
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record(st)
        ix.build_index(K_, V_)
        b.record(st)
        torch.cuda.synchronize()
        return a.elapsed_time(b)

    # one Lloyd round (assign + sort + means) = (build with 5 rounds - build with 1 round) / 4
    round_ms_layer = (build_ms(1, 5, K[0], V[0], init[0].contiguous()) - build_ms(1, 1, K[0], V[0], init[0].contiguous())) / 4
    round_ms_batched = (build_ms(L, 5, K, V, init.contiguous()) - build_ms(L, 1, K, V, init.contiguous())) / 4
    # the same on the transformed keys of Eq. 2 (one more coordinate: a ninth MFMA step per chain)
    round_ms_batched_tk = (build_ms(L, 5, K, V, init.contiguous(), 1) - build_ms(L, 1, K, V, init.contiguous(), 1)) / 4
    n_pages = batched.export()["n_pages"].cpu().numpy().astype(np.int64)              # [256]
    # two more copies of the batched index (same contents, other addresses): the timed loop rotates over
    # the three, 3 x 180 MB of lines touched per round against 256 MB of memory-side cache, so every
    # step finds its index evicted without a flush kernel between the steps
    rot = [batched]
    for _ in range(2):
        ix = IceIndex(L, H, G, max_tokens, s, C, kmeans_iters=T, init_idx=init.contiguous(), device=dev)
        ix.build_index(K, V)
        rot.append(ix)
    torch.cuda.synchronize()

    # ---------------------------------------------------------------- algorithmic bytes of one step
    # select: every live representative row (256 B) + the G query rows + the ids written;
    # attend: valid K and V rows of the selected pages + the fp32 outputs.
    flush = torch.zeros(1 << 28, dtype=torch.float32, device=dev)     # 1 GiB, read between timed steps
    ids_b = torch.empty((L, H, P), dtype=torch.int32, device=dev)
    ns_b = torch.empty((L, H), dtype=torch.int32, device=dev)
    out_b = torch.empty((L, H * G, D), dtype=torch.float32, device=dev)
    batched.select_attend(q, budget, ids_b, ns_b, out_b)
    torch.cuda.synchronize()
    exb = batched.export()
    fill = exb["page_fill"].cpu().numpy()
    ids_np, ns_np = ids_b.cpu().numpy().reshape(L * H, P), ns_b.cpu().numpy().reshape(L * H)
    sel_tokens = sum(int(fill[u, ids_np[u, :ns_np[u]]].sum()) for u in range(L * H))
    bytes_select = float(n_pages.sum()) * D * 2 + L * H * G * D * 2 + float(ns_np.sum()) * 4
    bytes_attend = sel_tokens * D * 2 * 2 + L * H * G * D * 4
    bytes_step = bytes_select + bytes_attend

    spread = [None]    # percentiles of the most recent timed() call

    def timed(fn, steps, warmup, cold=True):
        """ms per step.  All steps are enqueued without host round trips (flush, event, step, event),
        so the events bracket GPU execution of the step only; one synchronisation at the end."""
        for i in range(warmup):
            if cold:
                flush.sum()
            fn()
        torch.cuda.synchronize()
        evs = []
        for i in range(steps):
            if cold:
                flush.sum()                 # untimed: evicts L2 and the memory-side cache
            a, b = ev(), ev()
            a.record(st)
            fn()
            b.record(st)
            evs.append((a, b))
        torch.cuda.synchronize()
        ts = np.array([a.elapsed_time(b) for a, b in evs])
        spread[0] = {"median_us": float(np.median(ts)) * 1e3, "p10_us": float(np.percentile(ts, 10)) * 1e3,
                     "p90_us": float(np.percentile(ts, 90)) * 1e3}
        return float(ts.mean())

    cold = not args.warm
    # a plain copy of known size (256 MiB read, 256 MiB written): the reference dispatch against
    # which the HBM byte counters of a profiler run are scaled
    calib_src = flush[: 1 << 26]
    calib_dst = torch.empty_like(calib_src)
    torch.mul(calib_src, 1.0, out=calib_dst)
    # ---------------------------------------------------------------- batched: 256 units per launch set
    ms_flush = timed(lambda: batched.select_attend(q, budget, ids_b, ns_b, out_b), args.steps, args.warmup, cold)
    spread_batched = spread[0]
    # headline: `steps` launches back to back, rotating over the three index copies, one event pair
    # around the whole run (what a serving loop would see; the per-step brackets above each add the
    # event records and a dispatch gap to a 40 us kernel)
    if cold:
        for i in range(max(args.warmup, 3)):
            rot[i % 3].select_attend(q, budget, ids_b, ns_b, out_b)
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record(st)
        for i in range(args.steps):
            rot[i % 3].select_attend(q, budget, ids_b, ns_b, out_b)
        e1.record(st)
        torch.cuda.synchronize()
        ms_batched = e0.elapsed_time(e1) / args.steps
    else:
        ms_batched = ms_flush
    ms_sel = timed(lambda: ice_select(batched.handle, q, budget, ids_b, ns_b, None), args.steps, args.warmup, cold)
    ms_att = timed(lambda: batched.attend(q, ids_b, ns_b, out_b), args.steps, args.warmup, cold)

    # ---------------------------------------------------------------- hierarchical variant (clusters first)
    # the two-level form of the paper's top-down search: score the 512 centroids, keep the n_probe
    # best clusters, score only their pages; same launch shape and timing protocol as the headline
    n_probe = args.n_probe
    ids_h = torch.empty_like(ids_b)
    ns_h = torch.empty_like(ns_b)
    out_h = torch.empty_like(out_b)
    cl_h = torch.empty((L, H, n_probe), dtype=torch.int32, device=dev)
    hier = lambda ix: ice_select_hier(ix.handle, q, budget, n_probe, ids_h, ns_h, None, cl_h, out_h)
    for i in range(max(args.warmup, 3)):
        hier(rot[i % 3])
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record(st)
    for i in range(args.steps):
        hier(rot[i % 3])
    e1.record(st)
    torch.cuda.synchronize()
    ms_hier = e0.elapsed_time(e1) / args.steps
    hier(batched)
    torch.cuda.synchronize()
    pc = exb["page_cluster"].cpu().numpy()
    cl_np, idh_np, nsh_np = cl_h.cpu().numpy().reshape(L * H, n_probe), ids_h.cpu().numpy().reshape(L * H, P), ns_h.cpu().numpy().reshape(L * H)
    n_cand = sum(int(np.isin(pc[u, :n_pages[u]], cl_np[u][cl_np[u] >= 0]).sum()) for u in range(L * H))
    sel_tokens_h = sum(int(fill[u, idh_np[u, :nsh_np[u]]].sum()) for u in range(L * H))
    cpad = (C + 31) // 32 * 32
    bytes_hier = (L * H * (cpad * D * 2 + G * D * 2) + float(n_pages.sum()) * 4 + n_cand * D * 2 + float(nsh_np.sum()) * 4
                  + sel_tokens_h * D * 2 * 2 + L * H * G * D * 4)
    recall = float(np.mean([len(np.intersect1d(idh_np[u, :nsh_np[u]], ids_np[u, :ns_np[u]])) / max(1, ns_np[u])
                            for u in range(L * H)]))
    out_diff = float((out_h - out_b).abs().max().item())

    # ---------------------------------------------------------------- re-ranking by the best key (stage 3)
    # the 4P best pages by representative (of the kept clusters) are re-scored by their best key
    n_refine = 4 * P
    refine = lambda ix: ice_select_hier(ix.handle, q, budget, n_probe, ids_h, ns_h, None, cl_h, out_h, n_refine=n_refine)
    for i in range(max(args.warmup, 3)):
        refine(rot[i % 3])
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record(st)
    for i in range(args.steps):
        refine(rot[i % 3])
    e1.record(st)
    torch.cuda.synchronize()
    ms_refine = e0.elapsed_time(e1) / args.steps
    refine(batched)
    torch.cuda.synchronize()
    idr_np, nsr_np = ids_h.cpu().numpy().reshape(L * H, P), ns_h.cpu().numpy().reshape(L * H)

    # how many of the exact top-`budget` keys (by the group score q.k/||q||) the selected pages hold
    def key_recall(ids_sel, ns_sel, units=range(0, L * H, 8)):
        pos_all = exb["page_pos"]
        hits = []
        for u in units:
            l, h = divmod(u, H)
            qf = q[l].view(torch.bfloat16).float().reshape(H, G, D)[h]
            sc = (K[l, h].view(torch.bfloat16).float() @ (qf / qf.norm(dim=1, keepdim=True)).T).max(1).values
            top = set(torch.topk(sc, budget).indices.tolist())
            toks = pos_all[u, torch.from_numpy(ids_sel[u, :ns_sel[u]]).long().to(dev)].reshape(-1)
            hits.append(len(top & set(toks[toks >= 0].tolist())) / budget)
        return float(np.mean(hits))
    recall_keys = {"flat": key_recall(ids_np, ns_np), "hierarchical": key_recall(idh_np, nsh_np),
                   "refined": key_recall(idr_np, nsr_np)}

    # ---------------------------------------------------------------- with resident (sink + window) tokens
    # 16 sink + 256 window tokens per (layer, KV head) kept densely by the caller join the softmax
    n_res = 16 + 256
    g_res = torch.Generator(device="cpu").manual_seed(7)
    res_k = torch.randn((L, H, n_res, D), generator=g_res).to(torch.bfloat16).to(dev)
    res_v = torch.randn((L, H, n_res, D), generator=g_res).to(torch.bfloat16).to(dev)
    out_r = torch.empty_like(out_b)
    resident = lambda ix: ice_select_attend_resident(ix.handle, q, budget, res_k, res_v, n_res, ids_h, ns_h, out_r)
    for i in range(max(args.warmup, 3)):
        resident(rot[i % 3])
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record(st)
    for i in range(args.steps):
        resident(rot[i % 3])
    e1.record(st)
    torch.cuda.synchronize()
    ms_res = e0.elapsed_time(e1) / args.steps
    bytes_res = bytes_step + L * H * n_res * D * 2 * 2

    # ---------------------------------------------------------------- a selection reused by the following layers
    # the anchor layer's pages -> token positions -> attention over (here: the same) dense cache by position
    pos_t, n_tok_t = batched.selected_tokens(ids_b, ns_b)
    out_t = torch.empty_like(out_b)
    ms_tok = timed(lambda: batched.attend_tokens(q, K, V, pos_t, n_tok_t, out_t), args.steps, args.warmup, cold)
    tok_diff = float((out_t - out_b).abs().max().item())
    bytes_tok = float(n_tok_t.sum().item()) * D * 2 * 2 + float(n_tok_t.sum().item()) * 4 + L * H * G * D * 4

    # ---------------------------------------------------------------- one layer at a time, HIP graph of 32
    ids_l = [torch.empty((1, H, P), dtype=torch.int32, device=dev) for _ in range(L)]
    ns_l = [torch.empty((1, H), dtype=torch.int32, device=dev) for _ in range(L)]
    out_l = [torch.empty((1, H * G, D), dtype=torch.float32, device=dev) for _ in range(L)]
    q_l = [q[l:l + 1].contiguous() for l in range(L)]

    def seq_step():
        for l in range(L):
            per_layer[l].select_attend(q_l[l], budget, ids_l[l], ns_l[l], out_l[l])

    seq_step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        seq_step()
    graph.replay()
    torch.cuda.synchronize()
    same = all(torch.equal(out_l[l][0], out_b[l]) for l in range(L))
    ms_seq = timed(graph.replay, args.steps, args.warmup, cold)
    spread_seq = {k: v / L for k, v in spread[0].items()}

    # ---------------------------------------------------------------- what this machine reaches (measured peaks)
    # the library's own microbenchmarks: a streaming read of the 1 GiB flush buffer and a
    # register-resident MFMA loop; plus hipBLASLt's dense bf16 GEMM through torch.matmul (8192^3)
    sink = torch.zeros(1 << 19, dtype=torch.float32, device=dev)
    ice_debug_peak_read(flush, flush.numel() * 4, sink)
    mfma_flops = ice_debug_peak_mfma(sink, 2048)
    torch.cuda.synchronize()
    e0, e1, e2 = ev(), ev(), ev()
    e0.record(st)
    for _ in range(5):
        ice_debug_peak_read(flush, flush.numel() * 4, sink)
    e1.record(st)
    for _ in range(5):
        ice_debug_peak_mfma(sink, 2048)
    e2.record(st)
    torch.cuda.synchronize()
    stream_gbps = 5 * flush.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    mfma_loop_tflops = 5 * mfma_flops / (e1.elapsed_time(e2) * 1e-3) / 1e12
    ga = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
    gb = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
    gc = torch.matmul(ga, gb)
    torch.cuda.synchronize()
    e0.record(st)
    for _ in range(5):
        torch.matmul(ga, gb, out=gc)
    e1.record(st)
    torch.cuda.synchronize()
    gemm_tflops = 5 * 2.0 * 8192 ** 3 / (e0.elapsed_time(e1) * 1e-3) / 1e12
    del ga, gb, gc

    # ---------------------------------------------------------------- insertion (one token per unit)
    stream_in = datagen.DecodeStream(w, seed=w.seed)
    kk, vv, _ = stream_in.next()
    k1 = torch.from_numpy(np.tile(kk.view(np.int16), (L, 1, 1))).to(dev)
    v1 = torch.from_numpy(np.tile(vv.view(np.int16), (L, 1, 1))).to(dev)
    n_ins = 32
    e0, e1 = ev(), ev()
    batched.insert(k1, v1)
    torch.cuda.synchronize()
    e0.record(st)
    for _ in range(n_ins):
        batched.insert(k1, v1)
    e1.record(st)
    torch.cuda.synchronize()
    us_insert = e0.elapsed_time(e1) / n_ins * 1e3
    # a page of tokens at a time (tokens leaving the recent window): 16 per launch
    k16 = k1[:, :, None, :].expand(L, H, 16, D).contiguous()
    v16 = v1[:, :, None, :].expand(L, H, 16, D).contiguous()
    batched.insert_batch(k16, v16)
    torch.cuda.synchronize()
    e0.record(st)
    batched.insert_batch(k16, v16)
    batched.insert_batch(k16, v16)
    e1.record(st)
    torch.cuda.synchronize()
    us_insert16 = e0.elapsed_time(e1) / 2 * 1e3

    # ---------------------------------------------------------------- CPU oracle on the same step
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ice_oracle as orc
        o = orc.OracleIndex(L * H, G, s, C, max_tokens)
        for name in ("n_pages", "Kp", "Vp", "page_fill", "rep"):
            arr = exb[name].cpu().numpy()
            getattr(o, name)[...] = arr.view(np.uint16) if arr.dtype == np.int16 else arr
        qn = q_np.reshape(L * H, G, D)
        threads = orc.num_threads()
        t0 = time.time()
        oid, ons, _, _ = o.select(qn, budget)
        ref = o.attend(qn, oid, ons)
        t_all = time.time() - t0
        orc.set_num_threads(1)
        t0 = time.time()
        o.select(qn, budget)
        o.attend(qn, oid, ons)
        t_one = time.time() - t0
        orc.set_num_threads(threads)
        # one Lloyd round (exhaustive assign + means) of ONE unit of layer 0
        t0 = time.time()
        orc.lloyd(K0_np, init0_np, 1)
        t_round = time.time() - t0
        ids_match = bool(np.array_equal(oid, ids_np))
        err = float(np.abs(out_b.cpu().numpy().reshape(ref.shape) - ref).max())
        cpu = {"value": t_all / L * 1e6, "unit": "us/layer-step", "cores": threads, "kind": "oracle",
               "sample": "one full step: select+attend of all %d layers (%d units), fp64, OpenMP over units" % (L, L * H),
               "single_thread_us_per_layer_step": t_one / L * 1e6,
               "clustering_round_one_unit_s": t_round,
               "clustering_sample": "one Lloyd round of one (layer, KV head) unit, n=%d, C=%d, fp64, OpenMP over keys on %d threads" % (n, C, threads),
               "gpu_matches_oracle": {"page_ids_equal": ids_match, "attend_max_abs_err": err}}

    us_layer = ms_batched * 1e3 / L
    gbps = bytes_step / (ms_batched * 1e-3) / 1e9
    sel_gbps = bytes_select / (ms_sel * 1e-3) / 1e9
    line = {
        "metric": "select+attend us per layer-step (%dk ctx, %d-token budget)" % (n // 1024, budget),
        "value": us_layer, "unit": "us/layer-step",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_batched,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload + ": %d independent layers x (B=1, %d KV heads, GQA %d, d=128, n=%d, page %d, "
                               "%d clusters, budget %d), batched in one launch set of %d units; %s"
                               % (L, H, G, n, s, C, budget, L * H,
                                  "cold (steps rotate over three copies of the index, 540 MB, so none is cache resident)" if cold else "warm"),
                   "kmeans_iters": T},
        "effective_GBps": gbps,
        "bytes_per_step": bytes_step,
        "hbm_frac": gbps / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "kernel": "decode_step_kernel<4,16,%d> (score + top-P + attention in one launch), "
                                               "%d units, workgroups of 1024 threads (one per unit from 256 units on, "
                                               "else 256/units per unit)" % (4 if (max_tokens // s + C) <= 4096 else 16, L * H),
                     "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES if (args.workload, L) == ("cfg2", 32) else None, "algorithmic_bytes_per_launch": bytes_step,
                     "us_per_launch": ms_batched * 1e3,
                     "traffic_note": "rocprofv3 --pmc FETCH_SIZE x 2.0 (the counter reads half of a plain copy kernel's "
                                     "known bytes) + WRITE_SIZE x 1.0; see profiles/"},
        "select_only": {"us_per_launch": ms_sel * 1e3, "GBps": sel_gbps, "algorithmic_bytes_per_launch": bytes_select},
        "attend": {"us_per_launch": ms_att * 1e3, "GBps": bytes_attend / (ms_att * 1e-3) / 1e9,
                   "algorithmic_bytes_per_launch": bytes_attend},
        "hierarchical": {"n_probe": n_probe, "us_per_step": ms_hier * 1e3, "us_per_layer_step": ms_hier * 1e3 / L,
                         "algorithmic_bytes_per_step": bytes_hier, "GBps": bytes_hier / (ms_hier * 1e-3) / 1e9,
                         "candidate_pages_per_unit_mean": n_cand / (L * H),
                         "recall_of_flat_selection": recall, "attend_max_abs_diff_vs_flat": out_diff,
                         "how": "ice_select_hier (centroids -> kept clusters -> their pages -> top-P -> attention, one "
                                "launch), same rotation over three index copies as the headline"},
        "refined_by_best_key": {"n_probe": n_probe, "n_refine": n_refine, "us_per_step": ms_refine * 1e3,
                                "us_per_layer_step": ms_refine * 1e3 / L,
                                "top_key_recall": recall_keys,
                                "how": "ice_select_hier with n_refine = 4P: the 4P best pages by representative are re-ranked "
                                       "by their best key before the top P are attended; top_key_recall = share of the exact "
                                       "top-256 keys (q.k/||q||, max over the group) held by the selected pages, 32 sampled units"},
        "with_resident_tokens": {"n_resident": n_res, "us_per_step": ms_res * 1e3, "us_per_layer_step": ms_res * 1e3 / L,
                                 "algorithmic_bytes_per_step": bytes_res, "GBps": bytes_res / (ms_res * 1e-3) / 1e9,
                                 "how": "ice_select_attend_resident: 16 sink + 256 window tokens per unit in the same "
                                        "softmax as the selected pages; flat selection, same rotation"},
        "reuse_by_position": {"attend_tokens_us_per_step": ms_tok * 1e3, "algorithmic_bytes_per_step": bytes_tok,
                              "GBps": bytes_tok / (ms_tok * 1e-3) / 1e9,
                              "us_per_layer_step_anchor_every_3_layers": (ms_flush + 2 * ms_tok) * 1e3 / 3 / L,
                              "max_abs_diff_vs_page_attention": tok_diff,
                              "how": "ice_selected_tokens once, then ice_attend_tokens over the dense cache by token "
                                     "position (flush + one event pair per step, like flush_per_step); two of three "
                                     "layers skip the selection"},
        "sequential": {"us_per_layer_step": ms_seq * 1e3 / L, "GBps": bytes_step / (ms_seq * 1e-3) / 1e9,
                       "how": "HIP graph replay of 32 one-layer select+attend calls (8 units each)",
                       "bitwise_equal_to_batched": same},
        "clustering": {"build_ms_per_layer": build_ms_layer, "build_ms_batched_32_layers": build_ms_batched,
                       "lloyd_rounds": T,
                       "round_us_one_layer": round_ms_layer * 1e3, "round_us_batched_32_layers": round_ms_batched * 1e3,
                       "round_TFLOPs_one_layer": assign_flop_round / L / (round_ms_layer * 1e-3) / 1e12,
                       "round_TFLOPs_batched": assign_flop_round / (round_ms_batched * 1e-3) / 1e12,
                       "round_us_batched_transformed_keys": round_ms_batched_tk * 1e3,
                       "note": "a round is assign (MFMA) + counting sort + means; TFLOP/s counts the assign flops only, "
                               "so it is a lower bound on the assign kernel's own rate (see profiles/ for that)",
                       "assign_TFLOPs_lower_bound": assign_flop_round * T / (build_ms_batched * 1e-3) / 1e12,
                       "mfma_peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS},
        "measured_on_this_box": {"stream_read_GBps": stream_gbps, "mfma_loop_bf16_TFLOPs": mfma_loop_tflops,
                                 "hipblaslt_bf16_gemm_8192_TFLOPs": gemm_tflops,
                                 "value_frac_of_stream_read": gbps / stream_gbps,
                                 "round_batched_frac_of_mfma_loop": assign_flop_round / (round_ms_batched * 1e-3) / 1e12 / mfma_loop_tflops,
                                 "how": "ice_debug_peak_read over 1 GiB; ice_debug_peak_mfma (register operands, "
                                        "4 chains per wave, 32 waves per CU); torch.matmul bf16 8192^3"},
        "flush_per_step": {"us_per_step": ms_flush * 1e3,
                           "how": "same launch, one event pair per step, 1 GiB read between steps (untimed)"},
        "spread": {"batched_us_per_step": spread_batched, "sequential_us_per_layer_step": spread_seq},
        "insert": {"us_per_call_256_units": us_insert, "us_per_call_of_16_tokens_256_units": us_insert16},
        "pages_per_unit_mean": float(n_pages.mean()),
        "datagen_s": t_gen,
        "cpu_baseline": cpu,
        "paper_context": "paper reports whole-model TPOT 0.11 s on A100+64 CPU threads at 36k (Sec. 5.3.2); other hardware, context only",
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
