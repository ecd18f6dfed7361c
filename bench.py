#!/usr/bin/env python3
"""Benchmark of the IceCache hot path on one MI355X.

Headline workload (default, `--workload cfg2`): the Llama-3-8B-shaped layer of the benchmark
definition -- batch 1, 8 KV heads / 32 query heads, head_dim 128, context 32768, page_size 16, 512
clusters per KV head, token budget 256 -- for 32 independently seeded layers.  One "step" is one
decode token's select+attend over all 32 layers (256 units).  Printed value: microseconds per
layer-step with the 32 independent layers batched in one launch set; the one-layer-at-a-time figure
(HIP-graph replay of 32 launches) is reported beside it, together with the index build (clustering,
every stage timed by itself), insertion, the roofline of the dominant kernel and the CPU oracle
timed on the host cores.  The default run also measures the other four workloads of the benchmark
definition in compact form (`other_configs`: cfg1, cfg3, cfg4, cfg5 -- the last as the real
insert -> select -> attend loop), each with the oracle beside it; `--workload cfgN` prints one of
them as the line's own value.

All inputs are seeded synthetic data (datagen.py) resident in HBM before the timed region.  No timed
"cold" step may find its index in L2 or in the 256 MB memory-side cache: a cold loop rotates over as
many copies of the index as it takes to touch more than 600 MB of lines per round, with one event
pair around all steps; where that would take too many copies (cfg1, cfg5: a fraction of a MB per
step) every step is bracketed by its own event pair and an untimed 1 GiB read comes before it.
(Reading rather than writing the flush buffer leaves clean lines behind; dirty lines would add
write-back traffic to the timed kernel.)  Every figure labelled "cold" is therefore an HBM figure.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import datagen  # noqa: E402

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
D = 128
TRAFFIC_PROFILE = "profiles/decode_step_cfg2_hbm_counters.md"


def measured_traffic_bytes():
    """HBM bytes of one batched decode_step launch (fetch + write) as the committed counter summary
    states them (a line `traffic_kib_per_launch decode_step_cfg2_256_units = N`); None if absent."""
    try:
        text = open(os.path.join(ROOT, TRAFFIC_PROFILE)).read()
    except OSError:
        return None
    m = re.search(r"traffic_kib_per_launch\s+decode_step_cfg2_256_units\s*=\s*(\d+)", text)
    return int(m.group(1)) * 1024 if m else None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layers", type=int, default=32, help="independent layers batched in one launch (cfg2 only)")
    ap.add_argument("--kmeans-iters", type=int, default=10)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"],
                    help="cfg2 is the headline (and carries the other four in compact form); the others print their own line")
    ap.add_argument("--n-probe", type=int, default=0, help="clusters kept by the hierarchical variant (default n_clusters / 8)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--skip-others", action="store_true", help="cfg2 only: leave out the compact block of the other workloads")
    ap.add_argument("--warm", action="store_true", help="cfg2 only: skip the cache eviction between steps")
    return ap.parse_args()


def gen_layer(w, layer):
    K, V = datagen.keys_values(w, seed=w.seed + layer)
    return K[0], V[0], datagen.init_indices(w, seed=w.seed + layer)[0], datagen.queries(w, seed=w.seed + layer)[0]


class Clock:
    """Event timing on the stream the library's kernels are launched on."""

    def __init__(self, torch, dev):
        self.torch = torch
        self.st = torch.cuda.current_stream()
        self.flush = torch.zeros(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB, read between timed steps
        self.spread = None

    def ev(self):
        return self.torch.cuda.Event(enable_timing=True)

    def per_step(self, fn, steps, warmup, cold=True):
        """ms per step, one event pair per step, an untimed 1 GiB read before each cold step.  All steps
        are enqueued without host round trips; one synchronisation at the end."""
        torch = self.torch
        for _ in range(warmup):
            if cold:
                self.flush.sum()
            fn()
        torch.cuda.synchronize()
        evs = []
        for _ in range(steps):
            if cold:
                self.flush.sum()
            a, b = self.ev(), self.ev()
            a.record(self.st)
            fn()
            b.record(self.st)
            evs.append((a, b))
        torch.cuda.synchronize()
        ts = np.array([a.elapsed_time(b) for a, b in evs])
        self.spread = {"median_us": float(np.median(ts)) * 1e3, "p10_us": float(np.percentile(ts, 10)) * 1e3,
                       "p90_us": float(np.percentile(ts, 90)) * 1e3}
        return float(ts.mean())

    def back_to_back(self, fns, steps, warmup):
        """ms per step of `steps` calls issued back to back, rotating over fns, one event pair around all."""
        torch = self.torch
        for i in range(max(warmup, len(fns))):
            fns[i % len(fns)]()
        torch.cuda.synchronize()
        e0, e1 = self.ev(), self.ev()
        e0.record(self.st)
        for i in range(steps):
            fns[i % len(fns)]()
        e1.record(self.st)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    def once(self, fn, reps=1):
        torch = self.torch
        torch.cuda.synchronize()
        e0, e1 = self.ev(), self.ev()
        e0.record(self.st)
        for _ in range(reps):
            fn()
        e1.record(self.st)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps


def step_bytes(n_pages, ids_np, ns_np, fill, G):
    """Algorithmic bytes of one select+attend step: every live representative row (256 B) + the G query
    rows + the ids written; valid K and V rows of the selected pages + the fp32 outputs."""
    U = len(n_pages)
    sel_tokens = sum(int(fill[u, ids_np[u, :ns_np[u]]].sum()) for u in range(U))
    b_sel = float(n_pages.sum()) * D * 2 + U * G * D * 2 + float(ns_np.sum()) * 4
    b_att = sel_tokens * D * 2 * 2 + U * G * D * 4
    return b_sel, b_att


def stage_times(torch, clock, ix, K, V, reps=3):
    """us per kernel of the build's stages on a freshly built index (each re-run reproduces its output)."""
    from paper_2604_10539_amd import binding as b
    out = {}
    for name, stage in (("assign", b.ICE_STAGE_ASSIGN), ("sort", b.ICE_STAGE_SORT), ("means", b.ICE_STAGE_MEANS),
                        ("paginate", b.ICE_STAGE_PAGINATE)):
        b.ice_debug_rerun_stage(ix.handle, K, V, stage)
        out[name + "_us"] = clock.once(lambda: b.ice_debug_rerun_stage(ix.handle, K, V, stage), reps) * 1e3
    return out


def clustering_block(torch, clock, ix, K, V, T, build_ms, n, C, U):
    st = stage_times(torch, clock, ix, K, V)
    flop = 2.0 * n * C * D * U
    kv_bytes = float(U) * n * D * 2
    round_us = st["assign_us"] + st["sort_us"] + st["means_us"]
    return {
        "build_ms": build_ms, "lloyd_rounds": T, **st,
        "assign_TFLOPs": flop / (st["assign_us"] * 1e-6) / 1e12,
        "assign_frac_of_mfma_peak": flop / (st["assign_us"] * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "round_us": round_us, "round_TFLOPs": flop / (round_us * 1e-6) / 1e12,
        "round_frac_of_mfma_peak": flop / (round_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "means_GBps": kv_bytes / (st["means_us"] * 1e-6) / 1e9,
        "paginate_GBps": 4.0 * kv_bytes / (st["paginate_us"] * 1e-6) / 1e9,
        "paginate_frac_of_hbm_peak": 4.0 * kv_bytes / (st["paginate_us"] * 1e-6) / 1e9 / HBM_PEAK_GBPS,
        # what the build spends outside the timed stages: promotion of the initial centroids, the tail copies kept for
        # the insertions, resets, and the gaps between the launches (build time minus rounds and paginate)
        "init_and_rest_us": build_ms * 1e3 - T * round_us - st["paginate_us"],
        "how": "every stage re-run by itself on the built index (ice_debug_rerun_stage) between two events; assign counts "
               "2 n C d flop per unit; a round = assign + sort + means; means reads the keys once more (n d 2 B per unit), "
               "paginate reads K and V and writes both page tiles (4 n d 2 B per unit); init_and_rest_us = build - rounds - "
               "paginate (negative where the stages run faster inside the build, with the keys still cached, than alone)",
    }


# ------------------------------------------------------------------------------------------------
def compact_config(name, torch, dev, clock, args, stream_data=None):
    """One workload of the benchmark definition as its select+attend step (cfg5: as its decode loop), the
    index build, and the CPU oracle on the same step."""
    from paper_2604_10539_amd import IceIndex
    w = datagen.WORKLOADS[name]
    B, H, G, n, s, C, budget = w.batch, w.n_kv_heads, w.group_size, w.n_tokens, w.page_size, w.n_clusters, w.token_budget
    U, P, T = B * H, budget // s, args.kmeans_iters
    extra = w.decode_steps if w.decode_steps else 128
    max_tokens = n + extra
    t0 = time.time()
    K_np, V_np = datagen.keys_values(w, workers=16)
    init_np, q_np = datagen.init_indices(w), datagen.queries(w)
    t_gen = time.time() - t0
    K = torch.from_numpy(K_np.view(np.int16)).to(dev)
    V = torch.from_numpy(V_np.view(np.int16)).to(dev)
    init = torch.from_numpy(init_np).to(dev)
    q = torch.from_numpy(q_np.view(np.int16)).to(dev)

    def new_index():
        ix = IceIndex(B, H, G, max_tokens, s, C, kmeans_iters=T, init_idx=init, device=dev)
        ix.build_index(K, V)
        return ix

    first = new_index()
    build_ms = clock.once(lambda: first.build_index(K, V))
    ids = torch.empty((B, H, P), dtype=torch.int32, device=dev)
    ns = torch.empty((B, H), dtype=torch.int32, device=dev)
    out = torch.empty((B, H * G, D), dtype=torch.float32, device=dev)
    first.select_attend(q, budget, ids, ns, out)
    torch.cuda.synchronize()
    out0 = out.clone()
    ex = first.export()
    n_pages = ex["n_pages"].cpu().numpy().astype(np.int64)
    fill = ex["page_fill"].cpu().numpy()
    ids_np, ns_np = ids.cpu().numpy().reshape(U, P), ns.cpu().numpy().reshape(U)
    b_sel, b_att = step_bytes(n_pages, ids_np, ns_np, fill, G)
    b_step = b_sel + b_att
    clustering = clustering_block(torch, clock, first, K, V, T, build_ms, n, C, U)

    res = {"shape": "B=%d, %d KV heads, GQA %d, n=%d, page %d, %d clusters, budget %d: %d units, %.0f live pages per unit"
                    % (B, H, G, n, s, C, budget, U, float(n_pages.mean())),
           "algorithmic_bytes_per_step": b_step}
    # ---- the step, cold
    copies = int(np.ceil(600e6 / b_step))
    ws_gb = first.workspace.numel() / 1e9
    ms_flush = clock.per_step(lambda: first.select_attend(q, budget, ids, ns, out), args.steps, args.warmup, True)
    res["flush_per_step"] = {"us_per_step": ms_flush * 1e3, **clock.spread,
                             "how": "one event pair per step, untimed 1 GiB read before each"}
    ms = ms_flush
    res["timing"] = "flush_per_step (rotating over copies would take %d of them)" % copies
    if copies <= 40 and copies * ws_gb <= 60.0:
        rot = [first] + [new_index() for _ in range(copies - 1)]
        torch.cuda.synchronize()
        ms = clock.back_to_back([(lambda ix=ix: ix.select_attend(q, budget, ids, ns, out)) for ix in rot], max(args.steps, 2 * copies),
                                args.warmup)
        res["timing"] = "back to back over %d copies of the index (%.0f MB of lines per round), one event pair around all steps" % (
            copies, copies * b_step / 1e6)
        del rot
    res.update({"us_per_step": ms * 1e3, "GBps": b_step / (ms * 1e-3) / 1e9, "hbm_frac": b_step / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS})
    ms_warm = clock.back_to_back([lambda: first.select_attend(q, budget, ids, ns, out)], args.steps, args.warmup)
    res["warm_us_per_step"] = ms_warm * 1e3
    res["clustering"] = clustering
    # ---- the staged searches on the same index (cold: flush + one event pair per step)
    from paper_2604_10539_amd import binding
    n_probe = max(1, C // 8)
    ids_h, ns_h, out_h = torch.empty_like(ids), torch.empty_like(ns), torch.empty_like(out)
    try:
        ms_h = clock.per_step(lambda: binding.ice_select_hier(first.handle, q, budget, n_probe, ids_h, ns_h, None, None, out_h),
                              args.steps, args.warmup, True)
        rec2 = float(np.mean([len(np.intersect1d(ids_h.cpu().numpy().reshape(U, P)[u2, :ns_np[u2]], ids_np[u2, :ns_np[u2]])) / max(1, ns_np[u2])
                              for u2 in range(U)]))
        staged = {"two_levels": {"n_probe": n_probe, "us_per_step": ms_h * 1e3, "recall_of_flat_selection": rec2}}
        if C >= 64:
            n_top = min(256, max(8, int(round(np.sqrt(C) * 1.5))))
            n_probe_top = max(2, n_top // 4)
            t_top = clock.once(lambda: first.build_top_level(n_top, 3))
            ms_3 = clock.per_step(lambda: binding.ice_select_hier3(first.handle, q, budget, n_probe_top, n_probe, ids_h, ns_h, None, None,
                                                                    None, out_h), args.steps, args.warmup, True)
            rec3 = float(np.mean([len(np.intersect1d(ids_h.cpu().numpy().reshape(U, P)[u2, :ns_np[u2]], ids_np[u2, :ns_np[u2]])) / max(1, ns_np[u2])
                                  for u2 in range(U)]))
            staged["three_levels"] = {"n_top": n_top, "n_probe_top": n_probe_top, "n_probe": n_probe, "us_per_step": ms_3 * 1e3,
                                      "recall_of_flat_selection": rec3, "build_top_level_us": t_top * 1e3}
        staged["flat_flush_per_step_us"] = ms_flush * 1e3
        if name == "cfg3":
            # The same shapes on a nested mixture (the centres gather around 64 points): data with structure
            # above the clusters, which is what a third level can summarise; the plain mixture has none.
            wn = dataclasses.replace(w, n_super=64, super_spread=0.4, outlier_frac=0.0, seed=w.seed + 7)
            Kn_np, Vn_np = datagen.keys_values(wn, workers=16)
            Kn, Vn = torch.from_numpy(Kn_np.view(np.int16)).to(dev), torch.from_numpy(Vn_np.view(np.int16)).to(dev)
            qn = torch.from_numpy(datagen.queries(wn).view(np.int16)).to(dev)
            nix = IceIndex(B, H, G, max_tokens, s, C, kmeans_iters=T, init_idx=torch.from_numpy(datagen.init_indices(wn)).to(dev), device=dev)
            nix.build_index(Kn, Vn)
            nix.build_top_level(n_top, 3)
            ids_f, ns_f = torch.empty_like(ids), torch.empty_like(ns)
            ms_nf = clock.per_step(lambda: nix.select_attend(qn, budget, ids_f, ns_f, out_h), args.steps, args.warmup, True)
            ms_n2 = clock.per_step(lambda: binding.ice_select_hier(nix.handle, qn, budget, n_probe, ids_h, ns_h, None, None, out_h),
                                   args.steps, args.warmup, True)
            ids_2 = ids_h.cpu().numpy().reshape(U, P).copy()
            ms_n3 = clock.per_step(lambda: binding.ice_select_hier3(nix.handle, qn, budget, n_probe_top, n_probe, ids_h, ns_h, None, None,
                                                                     None, out_h), args.steps, args.warmup, True)
            idf, nsf = ids_f.cpu().numpy().reshape(U, P), ns_f.cpu().numpy().reshape(U)
            recall = lambda got: float(np.mean([len(np.intersect1d(got[u2, :nsf[u2]], idf[u2, :nsf[u2]])) / max(1, nsf[u2]) for u2 in range(U)]))
            staged["on_nested_mixture"] = {
                "data": "the same shapes, centres ~ one of 64 points + 0.4 N(0, I) instead of N(0, I)",
                "flat_us_per_step": ms_nf * 1e3, "two_levels_us_per_step": ms_n2 * 1e3, "two_levels_recall": recall(ids_2),
                "three_levels_us_per_step": ms_n3 * 1e3, "three_levels_recall": recall(ids_h.cpu().numpy().reshape(U, P))}
            del nix, Kn, Vn
        res["staged_search"] = staged
    except binding.IceError as e:
        res["staged_search"] = {"unsupported": str(e)}

    # ---- cfg5: the decode loop itself (Alg. 1 decode phase: insert -> select -> attend, one token per step)
    loop = None
    if w.decode_steps:
        ks_np, vs_np, qs_np = stream_data if stream_data is not None else datagen.DecodeStream(w).take(w.decode_steps)
        ks = torch.from_numpy(ks_np.view(np.int16)).to(dev)
        vs = torch.from_numpy(vs_np.view(np.int16)).to(dev)
        qs = torch.from_numpy(qs_np.view(np.int16)).to(dev)
        m = w.decode_steps
        a_ix, b_ix = new_index(), new_index()
        # the C ABI called directly with raw addresses: the host must not be what the loop waits for
        from paper_2604_10539_amd import binding
        lib, hs = binding.lib(), clock.st.cuda_stream
        kp, vp, qp = ks.data_ptr(), vs.data_ptr(), qs.data_ptr()
        kstep, qstep = U * D * 2, U * G * D * 2
        idp, nsp, outp = ids.data_ptr(), ns.data_ptr(), out.data_ptr()
        torch.cuda.synchronize()
        t0 = time.time()
        e0, e1 = clock.ev(), clock.ev()
        e0.record(clock.st)
        rc = 0
        for t in range(m):
            rc |= lib.ice_insert(a_ix.handle, kp + t * kstep, vp + t * kstep, hs)
            rc |= lib.ice_select_attend(a_ix.handle, qp + t * qstep, budget, idp, nsp, outp, hs)
        e1.record(clock.st)
        t_issue = time.time() - t0
        torch.cuda.synchronize()
        assert rc == 0, binding.ice_last_error()
        loop_ms = e0.elapsed_time(e1)

        def insert_only():
            r = 0
            for t in range(m):
                r |= lib.ice_insert(b_ix.handle, kp + t * kstep, vp + t * kstep, hs)
            assert r == 0
        ins_ms = clock.once(insert_only)
        np_end = a_ix.export()["n_pages"].cpu().numpy().astype(np.int64)
        ids_e, ns_e = ids.cpu().numpy().reshape(U, P), ns.cpu().numpy().reshape(U)
        b_sel_e, b_att_e = step_bytes(np_end, ids_e, ns_e, a_ix.export()["page_fill"].cpu().numpy(), G)
        b_loop = 0.5 * (b_step + b_sel_e + b_att_e) + U * (C * D * 2 + 2048)
        loop = {"steps": m, "us_per_step": loop_ms / m * 1e3, "insert_us_per_step": ins_ms / m * 1e3,
                "select_attend_us_per_step": (loop_ms - ins_ms) / m * 1e3,
                "host_issue_us_per_step": t_issue / m * 1e6,
                "algorithmic_bytes_per_step": b_loop, "GBps": b_loop / (loop_ms / m * 1e-3) / 1e9,
                "pages_per_unit_start_end": [float(n_pages.mean()), float(np_end.mean())],
                "how": "%d eager steps of ice_insert + ice_select_attend issued back to back on one stream, one event pair "
                       "around the loop (not a HIP graph: the token count that guards the capacity advances on the host "
                       "with every call); the index of one layer (%.0f MB touched per step) stays in the 256 MB cache, as "
                       "it would between the steps of a one-layer loop; insert alone is timed on a second copy; bytes = mean "
                       "of the first and last step plus the centroid scan and the appended rows" % (m, b_step / 1e6)}
        res["decode_loop"] = loop
        del a_ix, b_ix, ks, vs, qs

    # ---- CPU oracle on the same step
    if not args.no_cpu_baseline:
        from oracle import ice_oracle as orc
        o = orc.OracleIndex(U, G, s, C, max_tokens)
        for nm in ("n_pages", "Kp", "Vp", "page_fill", "rep", "page_cluster", "cluster_tail", "cluster_cnt", "cluster_sum", "centroid",
                   "page_sum", "page_pos"):
            arr = ex[nm].cpu().numpy()
            getattr(o, nm)[...] = arr.view(np.uint16) if arr.dtype == np.int16 else arr
        o.n_tokens[:] = n
        qn = q_np.reshape(U, G, D)
        threads = orc.num_threads()
        t0 = time.time()
        oid, ons, _, _ = o.select(qn, budget)
        ref = o.attend(qn, oid, ons)
        t_step = time.time() - t0
        t0 = time.time()
        orc.lloyd(K_np.reshape(U, n, D)[0], init_np.reshape(U, C)[0], 1)
        t_round = time.time() - t0
        cpu = {"us_per_step": t_step * 1e6, "cores": threads, "kind": "oracle",
               "sample": "one full step (select + attend of all %d units), fp64, OpenMP over units" % U,
               "clustering_round_one_unit_s": t_round,
               "clustering_sample": "one Lloyd round of ONE unit (one KV head of one sequence), n=%d, C=%d, OpenMP over keys" % (n, C),
               "gpu_matches_oracle": {"page_ids_equal": bool(np.array_equal(oid, ids_np)),
                                      "attend_max_abs_err": float(np.abs(out0.cpu().numpy().reshape(ref.shape) - ref).max())}}
        if w.decode_steps:
            ks_np, vs_np, qs_np = stream_data if stream_data is not None else datagen.DecodeStream(w).take(32)
            t0 = time.time()
            for t in range(32):
                o.insert(ks_np[t], vs_np[t])
                oi, on, _, _ = o.select(qs_np[t].reshape(U, G, D), budget)
                o.attend(qs_np[t].reshape(U, G, D), oi, on)
            cpu["decode_loop_us_per_step"] = (time.time() - t0) / 32 * 1e6
            cpu["decode_loop_sample"] = "the first 32 steps of the loop (insert + select + attend)"
        res["cpu_baseline"] = cpu
    res["datagen_s"] = t_gen
    del first, K, V
    torch.cuda.empty_cache()
    return res


# ------------------------------------------------------------------------------------------------
def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every unit is independent; more GPUs would just "
              "take disjoint heads or sequences); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    # the decode stream of cfg5 is drawn on forked processes, before this process touches the GPU
    stream5 = None
    if args.workload == "cfg5" or (args.workload == "cfg2" and not args.skip_others):
        w5 = datagen.WORKLOADS["cfg5"]
        stream5 = datagen.DecodeStream(w5).take(w5.decode_steps, workers=16)
    import torch
    from paper_2604_10539_amd import (IceIndex, ice_debug_peak_mfma, ice_debug_peak_read, ice_select, ice_select_attend_resident,
                                      ice_select_hier)

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    clock = Clock(torch, dev)
    st, ev, flush = clock.st, clock.ev, clock.flush

    if args.workload != "cfg2":
        r = compact_config(args.workload, torch, dev, clock, args, stream5)
        w = datagen.WORKLOADS[args.workload]
        loop = r.get("decode_loop")
        value = loop["us_per_step"] if loop else r["us_per_step"]
        gb = loop["GBps"] if loop else r["GBps"]
        cpu = r.pop("cpu_baseline", None)
        line = {"metric": "select+attend us per step (%dk ctx, %d-token budget)%s" % (w.n_tokens // 1024, w.token_budget,
                                                                                     ", with the insertion of the new token" if loop else ""),
                "value": value, "unit": "us/step", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                "ms_per_step": value * 1e-3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
                "dtype": "bf16", "data": "synthetic",
                "config": {"workload": args.workload + ": " + r["shape"] + "; " + (loop["how"] if loop else r["timing"]),
                           "kmeans_iters": args.kmeans_iters},
                "roofline": {"bound": "hbm", "achieved": gb, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gb / HBM_PEAK_GBPS,
                             "traffic": None, "algorithmic_bytes_per_launch": (loop or r)["algorithmic_bytes_per_step"],
                             "kernel": "decode_step_kernel (score + top-P + attention)" + (" after insert_kernel" if loop else "")},
                "cpu_baseline": None if cpu is None else {"value": cpu.get("decode_loop_us_per_step", cpu["us_per_step"]), "unit": "us/step",
                                                          **{k: v for k, v in cpu.items() if k != "us_per_step"}},
                "details": r}
        print(json.dumps(line))
        return

    w = dataclasses.replace(datagen.WORKLOADS["cfg2"], batch=1)
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

    # ---------------------------------------------------------------- index build (clustering + paging)
    # (a) one index per layer (B=1, 8 units): the one-layer-at-a-time decode path
    per_layer = [IceIndex(1, H, G, max_tokens, s, C, kmeans_iters=T, init_idx=init[l].contiguous(), device=dev)
                 for l in range(L)]
    per_layer[0].build_index(K[0], V[0])          # warm-up of every build kernel
    build_ms_layer = clock.once(lambda: [per_layer[l].build_index(K[l], V[l]) for l in range(L)]) / L
    clustering_one_layer = clustering_block(torch, clock, per_layer[0], K[0], V[0], T, build_ms_layer, n, C, H)
    # (b) all layers as one batch of 256 units: the batched decode path
    batched = IceIndex(L, H, G, max_tokens, s, C, kmeans_iters=T, init_idx=init.contiguous(), device=dev)
    build_ms_batched = clock.once(lambda: batched.build_index(K, V))
    clustering_batched = clustering_block(torch, clock, batched, K, V, T, build_ms_batched, n, C, L * H)
    assign_flop_round = 2.0 * n * C * D * H * L

    def build_ms(layers_, T_, K_, V_, init_, geometry=0):
        ix = IceIndex(layers_, H, G, max_tokens, s, C, kmeans_iters=T_, init_idx=init_, device=dev, geometry=geometry)
        ix.build_index(K_, V_)
        return clock.once(lambda: ix.build_index(K_, V_))

    # one Lloyd round on the transformed keys of Eq. 2 (one more coordinate: a ninth MFMA step per chain)
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
    ids_b = torch.empty((L, H, P), dtype=torch.int32, device=dev)
    ns_b = torch.empty((L, H), dtype=torch.int32, device=dev)
    out_b = torch.empty((L, H * G, D), dtype=torch.float32, device=dev)
    batched.select_attend(q, budget, ids_b, ns_b, out_b)
    torch.cuda.synchronize()
    exb = batched.export()
    fill = exb["page_fill"].cpu().numpy()
    ids_np, ns_np = ids_b.cpu().numpy().reshape(L * H, P), ns_b.cpu().numpy().reshape(L * H)
    bytes_select, bytes_attend = step_bytes(n_pages, ids_np, ns_np, fill, G)
    bytes_step = bytes_select + bytes_attend
    out_fused = out_b.clone()                     # the fused step's own output (out_b is reused below)

    cold = not args.warm
    timed = clock.per_step
    # a plain copy of known size (256 MiB read, 256 MiB written): the reference dispatch against
    # which the HBM byte counters of a profiler run are scaled
    calib_src = flush[: 1 << 26]
    calib_dst = torch.empty_like(calib_src)
    torch.mul(calib_src, 1.0, out=calib_dst)
    # ---------------------------------------------------------------- batched: 256 units per launch set
    ms_flush = timed(lambda: batched.select_attend(q, budget, ids_b, ns_b, out_b), args.steps, args.warmup, cold)
    spread_batched = clock.spread
    # headline: `steps` launches back to back, rotating over the three index copies, one event pair
    # around the whole run (what a serving loop would see; the per-step brackets above each add the
    # event records and a dispatch gap to a 40 us kernel)
    if cold:
        ms_batched = clock.back_to_back([(lambda ix=ix: ix.select_attend(q, budget, ids_b, ns_b, out_b)) for ix in rot], args.steps, args.warmup)
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
    ms_hier = clock.back_to_back([(lambda ix=ix: hier(ix)) for ix in rot], args.steps, args.warmup)
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
    out_diff = float((out_h - out_fused).abs().max().item())

    # ---------------------------------------------------------------- re-ranking by the best key (stage 3)
    # the 4P best pages by representative (of the kept clusters) are re-scored by their best key
    n_refine = 4 * P
    refine = lambda ix: ice_select_hier(ix.handle, q, budget, n_probe, ids_h, ns_h, None, cl_h, out_h, n_refine=n_refine)
    ms_refine = clock.back_to_back([(lambda ix=ix: refine(ix)) for ix in rot], args.steps, args.warmup)
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
    ms_res = clock.back_to_back([(lambda ix=ix: resident(ix)) for ix in rot], args.steps, args.warmup)
    bytes_res = bytes_step + L * H * n_res * D * 2 * 2

    # ---------------------------------------------------------------- a selection reused by the following layers
    # the anchor layer's pages -> token positions -> attention over (here: the same) dense cache by position
    batched.select_attend(q, budget, ids_b, ns_b, out_b)
    pos_t, n_tok_t = batched.selected_tokens(ids_b, ns_b)
    out_t = torch.empty_like(out_b)
    ms_tok = timed(lambda: batched.attend_tokens(q, K, V, pos_t, n_tok_t, out_t), args.steps, args.warmup, cold)
    tok_diff = float((out_t - out_fused).abs().max().item())
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
    # same ids and, since both forms attend in rank order with one workgroup per unit, the same output bits
    same_ids = all(torch.equal(ids_l[l][0], ids_b[l]) for l in range(L))
    same_out = all(torch.equal(out_l[l][0], out_fused[l]) for l in range(L))
    ms_seq = timed(graph.replay, args.steps, args.warmup, cold)
    spread_seq = {k: v / L for k, v in clock.spread.items()}
    # one layer's own bytes (the per-layer indices hold the same pages as the batched one)
    ms_one = timed(lambda: per_layer[0].select_attend(q_l[0], budget, ids_l[0], ns_l[0], out_l[0]), args.steps, args.warmup, cold)

    # ---------------------------------------------------------------- what this machine reaches (measured peaks)
    # the library's own microbenchmarks: a streaming read of the 1 GiB flush buffer and a
    # register-resident MFMA loop; plus hipBLASLt's dense bf16 GEMM through torch.matmul (8192^3)
    sink = torch.zeros(1 << 19, dtype=torch.float32, device=dev)
    ice_debug_peak_read(flush, flush.numel() * 4, sink)
    mfma_flops = ice_debug_peak_mfma(sink, 2048)
    stream_gbps = flush.numel() * 4 / (clock.once(lambda: ice_debug_peak_read(flush, flush.numel() * 4, sink), 5) * 1e-3) / 1e9
    mfma_loop_tflops = mfma_flops / (clock.once(lambda: ice_debug_peak_mfma(sink, 2048), 5) * 1e-3) / 1e12
    ga = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
    gb = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
    gc = torch.matmul(ga, gb)
    gemm_tflops = 2.0 * 8192 ** 3 / (clock.once(lambda: torch.matmul(ga, gb, out=gc), 5) * 1e-3) / 1e12
    del ga, gb, gc

    # ---------------------------------------------------------------- insertion
    # 32 + 3 x 16 consecutive tokens of every layer's own decode stream (seeded like the layer's keys, so
    # the tokens come from the distribution the layer was clustered on), one per launch and a page of 16 per
    # launch; the C ABI is called with raw addresses so that the host is not what the launches wait for
    from paper_2604_10539_amd import binding
    ins_ix = rot[2]          # (a copy of the index: the one the oracle is compared with stays as built)
    with ThreadPoolExecutor(max_workers=min(16, L)) as ex:
        taken = list(ex.map(lambda l: datagen.DecodeStream(w, seed=w.seed + l).take(32 + 3 * 16)[:2], range(L)))
    k_np = np.stack([t[0][:, 0] for t in taken], 1)                             # [80, L, H, D]
    v_np = np.stack([t[1][:, 0] for t in taken], 1)
    tile = lambda a: torch.from_numpy(np.ascontiguousarray(a.view(np.int16).transpose(1, 2, 0, 3))).to(dev)   # -> [L, H, m, D]
    k1, v1 = tile(k_np[:32]), tile(v_np[:32])                                   # token t at [:, :, t]
    k1 = k1.permute(2, 0, 1, 3).contiguous()                                    # [32, L, H, D]: one launch's keys contiguous
    v1 = v1.permute(2, 0, 1, 3).contiguous()
    k16 = [tile(k_np[32 + 16 * r:48 + 16 * r]) for r in range(3)]               # [L, H, 16, D] each
    v16 = [tile(v_np[32 + 16 * r:48 + 16 * r]) for r in range(3)]
    lib_raw, hs = binding.lib(), clock.st.cuda_stream
    step1 = L * H * D * 2

    def insert_singles(lo, hi):
        r = 0
        for t in range(lo, hi):
            r |= lib_raw.ice_insert(ins_ix.handle, k1.data_ptr() + t * step1, v1.data_ptr() + t * step1, hs)
        assert r == 0, binding.ice_last_error()
    insert_singles(0, 8)
    us_insert = clock.once(lambda: insert_singles(8, 32)) / 24 * 1e3
    ins_ix.insert_batch(k16[0], v16[0])

    def insert_pages():
        r = 0
        for i in (1, 2):
            r |= lib_raw.ice_insert_batch(ins_ix.handle, k16[i].data_ptr(), v16[i].data_ptr(), 16, hs)
        assert r == 0, binding.ice_last_error()
    us_insert16 = clock.once(insert_pages) / 2 * 1e3
    # the unfavourable case: every layer is given layer 0's tokens, which for the other 31 layers come from a
    # foreign distribution and crowd into a few clusters (most tokens of a launch then depend on each other)
    kf = torch.from_numpy(np.ascontiguousarray(np.tile(k_np[32:48, :1].view(np.int16), (1, L, 1, 1)).transpose(1, 2, 0, 3))).to(dev)
    vf = torch.from_numpy(np.ascontiguousarray(np.tile(v_np[32:48, :1].view(np.int16), (1, L, 1, 1)).transpose(1, 2, 0, 3))).to(dev)
    us_insert16_foreign = clock.once(lambda: ins_ix.insert_batch(kf, vf)) * 1e3

    # ---------------------------------------------------------------- CPU oracle on the same step
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ice_oracle as orc
        o = orc.OracleIndex(L * H, G, s, C, max_tokens)
        for name in ("n_pages", "Kp", "Vp", "page_fill", "rep"):
            arr = exb[name].cpu().numpy()
            getattr(o, name)[...] = arr.view(np.uint16) if arr.dtype == np.int16 else arr
        o.n_pages[...] = n_pages
        o.page_fill[...] = fill
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
        err = float(np.abs(out_fused.cpu().numpy().reshape(ref.shape) - ref).max())
        cpu = {"value": t_all / L * 1e6, "unit": "us/layer-step", "cores": threads, "kind": "oracle",
               "sample": "one full step: select+attend of all %d layers (%d units), fp64, OpenMP over units" % (L, L * H),
               "single_thread_us_per_layer_step": t_one / L * 1e6,
               "clustering_round_one_unit_s": t_round,
               "clustering_sample": "one Lloyd round of one (layer, KV head) unit, n=%d, C=%d, fp64, OpenMP over keys on %d threads" % (n, C, threads),
               "gpu_matches_oracle": {"page_ids_equal": ids_match, "attend_max_abs_err": err}}

    # free the headline's memory, then the other four workloads in compact form
    del per_layer, batched, rot, K, V, exb, graph
    torch.cuda.empty_cache()
    others = None
    if not args.skip_others:
        others = {}
        for name in ("cfg1", "cfg3", "cfg4", "cfg5"):
            others[name] = compact_config(name, torch, dev, clock, args, stream5 if name == "cfg5" else None)

    traffic = measured_traffic_bytes() if L == 32 else None
    us_layer = ms_batched * 1e3 / L
    gbps = bytes_step / (ms_batched * 1e-3) / 1e9
    sel_gbps = bytes_select / (ms_sel * 1e-3) / 1e9
    line = {
        "metric": "select+attend us per layer-step (%dk ctx, %d-token budget)" % (n // 1024, budget),
        "value": us_layer, "unit": "us/layer-step",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_batched,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg2: %d independent layers x (B=1, %d KV heads, GQA %d, d=128, n=%d, page %d, "
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
                     "traffic": traffic, "algorithmic_bytes_per_launch": bytes_step,
                     "us_per_launch": ms_batched * 1e3,
                     "traffic_note": "read at run time from " + TRAFFIC_PROFILE + " (two rocprofv3 --pmc runs of this command: "
                                     "FETCH_SIZE x 2.0, the counter reads half of a plain copy kernel's known bytes, + WRITE_SIZE x 1.0); "
                                     "that file names the commit it was measured at"},
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
                       "hbm_frac": bytes_step / (ms_seq * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                       "one_layer_alone_us": ms_one * 1e3,
                       "how": "HIP graph replay of 32 one-layer select+attend calls (8 units each); one_layer_alone_us = one such "
                              "call between its own event pair after the flush",
                       "page_ids_equal_to_batched": same_ids, "output_bits_equal_to_batched": same_out},
        "clustering": {"batched_32_layers": clustering_batched, "one_layer": clustering_one_layer,
                       "round_us_batched_transformed_keys": round_ms_batched_tk * 1e3,
                       "assign_TFLOPs_lower_bound_from_build": assign_flop_round * T / (build_ms_batched * 1e-3) / 1e12,
                       "mfma_peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS},
        "measured_on_this_box": {"stream_read_GBps": stream_gbps, "mfma_loop_bf16_TFLOPs": mfma_loop_tflops,
                                 "hipblaslt_bf16_gemm_8192_TFLOPs": gemm_tflops,
                                 "value_frac_of_stream_read": gbps / stream_gbps,
                                 "assign_batched_frac_of_mfma_loop": clustering_batched["assign_TFLOPs"] / mfma_loop_tflops,
                                 "how": "ice_debug_peak_read over 1 GiB; ice_debug_peak_mfma (register operands, "
                                        "4 chains per wave, 32 waves per CU); torch.matmul bf16 8192^3"},
        "flush_per_step": {"us_per_step": ms_flush * 1e3,
                           "how": "same launch, one event pair per step, 1 GiB read between steps (untimed)"},
        "spread": {"batched_us_per_step": spread_batched, "sequential_us_per_layer_step": spread_seq},
        "insert": {"us_per_call_256_units": us_insert, "us_per_call_of_16_tokens_256_units": us_insert16,
                   "us_per_call_of_16_crowding_tokens_256_units": us_insert16_foreign,
                   "how": "tokens of each layer's own decode stream, 24 single-token launches and 2 launches of 16 tokens "
                          "issued back to back between two events; crowding: layer 0's tokens given to every layer (foreign to "
                          "31 of them: most tokens of a launch land in the same few clusters and are settled one after the other)"},
        "pages_per_unit_mean": float(n_pages.mean()),
        "datagen_s": t_gen,
        "cpu_baseline": cpu,
        "other_configs": others,
        "paper_context": "paper reports whole-model TPOT 0.11 s on A100+64 CPU threads at 36k (Sec. 5.3.2); other hardware, context only",
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
