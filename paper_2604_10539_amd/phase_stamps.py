"""Where the time goes inside the decode-step and insertion kernels: in-kernel time stamps.

    python -m paper_2604_10539_amd.phase_stamps --build      (anywhere: compiles the stamped variant)
    python -m paper_2604_10539_amd.phase_stamps              (on the GPU: runs it and prints the tables)

The stamps are compiled in only with -DICE_PROF (csrc/ice_prof.h); this module builds that variant
into _build/prof/ beside the product library, which it never touches, loads it instead of the
product library, runs config 2 (one layer = 8 units, and 32 layers = 256 units) with a cold index,
and prints the phases of the workgroup that finishes a unit.  Times are microseconds after the
wave's first stamp; a stamp is taken by thread 0 of unit 0's workgroup (decode: of the workgroup
that is last to deliver its scores), so they are one workgroup's view, not a chip-wide average; the
per-unit table gives the spread over all units."""
from __future__ import annotations

import argparse
import ctypes
import os
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
PROF_DIR = os.path.join(ROOT, "_build", "prof")
PROF_LIB = os.path.join(PROF_DIR, "libicecache_prof.so")

# stamp index -> what has happened when it is taken (decode_step_kernel)
DECODE = [(0, "wave started"), (14, "own chunk scored"), (2, "last workgroup holds every score of the unit"),
          (3, "threshold known"), (4, "candidates listed"), (5, "pages ranked, ids written"), (6, "attention: tiles requested"),
          (7, "output written")]
INSERT_ONE = [(40, "wave started"), (41, "first barrier (LDS only)"), (45, "tiles in LDS"), (46, "dot products done"),
              (47, "wave's best row known"), (42, "state of that row requested"), (43, "waves have met"),
              (49, "cluster moved"), (44, "row appended")]
INSERT_BATCH = [(32, "wave started"), (33, "D[t][c] written"), (34, "barrier"), (35, "guess: state fetched, move and its dot products worked out"),
                (36, "barrier"), (37, "settled"), (38, "barrier"), (53, "own moves stored"), (55, "rows appended")]


def build() -> str:
    from .build import build_library
    os.makedirs(PROF_DIR, exist_ok=True)
    return build_library(extra_flags=("-DICE_PROF",), lib_path=PROF_LIB, obj_dir=os.path.join(PROF_DIR, "obj"))


def _stamps(lib, n=64):
    buf = (ctypes.c_longlong * n)()
    assert lib.ice_debug_prof_decode(buf, n) == 0
    return list(buf)


def _table(title, names, runs):
    print("\n### %s\n" % title)
    print("| after | " + " | ".join("run %d" % (i + 1) for i in range(len(runs))) + " |")
    print("|---|" + "---|" * len(runs))
    for idx, what in names:
        cell = lambda r: "%.2f" % ((r[idx] - r[names[0][0]]) / 100.0) if r[idx] >= r[names[0][0]] else "-"   # (-: not reached by the stamping thread)
        print("| %s | " % what + " | ".join(cell(r) for r in runs) + " |")


def run() -> None:
    import numpy as np
    import torch
    if not os.path.exists(PROF_LIB):
        build()
    from . import binding
    binding.LIB_PATH = PROF_LIB
    sys.path.insert(0, ROOT)
    import datagen
    from . import IceIndex
    lib = binding.lib()
    w = datagen.WORKLOADS["cfg2"]
    dev = "cuda:0"
    up = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)
    flush = torch.zeros(1 << 28, dtype=torch.float32, device=dev)

    def cold():
        flush.sum()
        torch.cuda.synchronize()

    for layers in (1, 32):
        gen = [(datagen.keys_values(w, seed=w.seed + l), datagen.init_indices(w, seed=w.seed + l)[0],
                datagen.queries(w, seed=w.seed + l)[0], datagen.DecodeStream(w, seed=w.seed + l).take(34)) for l in range(layers)]
        K = up(np.stack([g[0][0][0] for g in gen]))
        V = up(np.stack([g[0][1][0] for g in gen]))
        init, q = up(np.stack([g[1] for g in gen])), up(np.stack([g[2] for g in gen]))
        ks = np.stack([g[3][0][:, 0] for g in gen], 1)   # [34, layers, H, D]
        vs = np.stack([g[3][1][:, 0] for g in gen], 1)
        ix = IceIndex(layers, w.n_kv_heads, w.group_size, w.n_tokens + 64, w.page_size, w.n_clusters, kmeans_iters=4, init_idx=init, device=dev)
        ix.build_index(K, V)
        U = layers * w.n_kv_heads
        print("\n## config 2, %d layer%s in one launch (%d units)" % (layers, "" if layers == 1 else "s", U))
        runs, per_unit = [], None
        ix.select_attend(q, w.token_budget)
        for _ in range(3):
            cold()
            ix.select_attend(q, w.token_budget)
            torch.cuda.synchronize()
            runs.append(_stamps(lib))
        _table("decode step (ice_select_attend), cold index: unit 0", DECODE, runs)
        buf = (ctypes.c_longlong * (64 + 4096))()
        lib.ice_debug_prof_decode(buf, 64 + 4096)
        t = np.array(buf[64:64 + 4 * min(U, 1024)], dtype=np.int64).reshape(-1, 4)
        t = (t - t[:, 0].min()) / 100.0
        print("\nper unit (us after the first unit's start): " + "; ".join(
            "%s median %.2f, max %.2f" % (nm, np.median(t[:, c]), t[:, c].max())
            for nm, c in (("scores complete", 1), ("pages ranked", 2), ("output written", 3))))
        runs = []
        for r in range(3):
            cold()
            ix.insert(up(ks[r]), up(vs[r]))
            torch.cuda.synchronize()
            runs.append(_stamps(lib))
        _table("one token (ice_insert), cold index: unit 0 (the last two rows only when wave 0 is the wave whose row wins)", INSERT_ONE, runs)
        runs = []
        for r in range(2):
            kb = up(np.ascontiguousarray(ks[3 + 16 * r:19 + 16 * r].transpose(1, 2, 0, 3)))
            vb = up(np.ascontiguousarray(vs[3 + 16 * r:19 + 16 * r].transpose(1, 2, 0, 3)))
            cold()
            ix.insert_batch(kb, vb)
            torch.cuda.synchronize()
            runs.append(_stamps(lib))
        _table("16 tokens (ice_insert_batch), cold index: unit 0", INSERT_BATCH, runs)
        del ix, K, V


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--build", action="store_true", help="only compile the stamped variant")
    a = ap.parse_args()
    if a.build:
        print(build())
    else:
        run()
