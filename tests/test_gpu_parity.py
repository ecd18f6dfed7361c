"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same seeded
inputs.  Integer results (tables, page ids, bit copies, ordered-fp32 quantities) must be bit-exact;
floating-point decisions may differ only inside a stated tie band, which is counted and printed;
attention must agree within max-abs 2e-3 (bf16 inputs, fp32 accumulation)."""
import math

import numpy as np
import pytest
import torch

import datagen
from datagen import bf16_bits_to_f32 as widen, f32_to_bf16_bits as narrow
from oracle import ice_oracle as orc
from tests.util import D, STATE_FIELDS, down, export_np, oracle_arrays_to_device, oracle_from_export, up, valid_slot_mask

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3        # contract: max-abs on bf16 inputs with fp32 accumulation
ATTN_EXPECTED = 2e-4   # what fp32 accumulation actually delivers; a regression guard
SCORE_TIE = 1e-5       # ties within 1e-5 (relative to max(1, |score|)) are reported, not failed
U2 = 2.0 ** -24        # fp32 unit roundoff


def _mk(w, T=3, extra=0, init=True, seed=0):
    from paper_2604_10539_amd import IceIndex
    K, V = datagen.keys_values(w)
    idx = datagen.init_indices(w)
    ix = IceIndex(w.batch, w.n_kv_heads, w.group_size, w.n_tokens + extra, w.page_size, w.n_clusters,
                  kmeans_iters=T, seed=seed, init_idx=up(idx) if init else None)
    U = w.batch * w.n_kv_heads
    return ix, K.reshape(U, w.n_tokens, D), V.reshape(U, w.n_tokens, D), idx.reshape(U, w.n_clusters)


def _assign_band(K, mub):
    """Rigorous bound on |fp32 objective - exact objective| for one unit: the objective is a chain of
    d+1 fp32 additions of exact products seeded with -w/2, then doubled."""
    kf, mf = widen(K).astype(np.float64), widen(mub).astype(np.float64)
    w = (mf ** 2).sum(1)
    mag = 0.5 * w.max() + np.linalg.norm(kf, axis=1) * np.linalg.norm(mf, axis=1).max()
    return 2.0 * (D + 2) * U2 * mag * 2.0


def _check_assign(K, mub, a_gpu, label):
    """GPU choice must be optimal within the tie band; returns the number of rows that differ."""
    a_ref, best, second = orc.assign(K, mub)
    kf, mf = widen(K).astype(np.float64), widen(mub).astype(np.float64)
    obj_gpu = (mf[a_gpu] ** 2).sum(1) - 2.0 * (kf * mf[a_gpu]).sum(1)
    band = _assign_band(K, mub)
    diff = np.nonzero(a_gpu != a_ref)[0]
    assert np.all(obj_gpu - best <= band), "%s: a GPU assignment is worse than the optimum beyond the tie band" % label
    print("[assign %s] %d of %d rows differ from the oracle, all inside the tie band (max band %.2e)"
          % (label, len(diff), len(a_ref), band.max()))
    assert len(diff) <= max(2, len(a_ref) // 500), "%s: too many near-tie flips" % label
    return len(diff)


# ----------------------------------------------------------------------------------------- assign
@pytest.mark.parametrize("n,C", [(1000, 24), (4096, 32), (5000, 100), (3001, 512), (2100, 700), (4099, 2048), (333, 1)])
def test_debug_assign_matches_exhaustive_search(n, C):
    from paper_2604_10539_amd import IceIndex
    rng = np.random.default_rng(n + C)
    w = datagen.small(n_tokens=n, n_clusters=C, n_kv_heads=2, n_components=max(4, C // 2))
    K, _ = datagen.keys_values(w)
    K = K.reshape(2, n, D)
    mub = np.stack([K[u][rng.choice(n, C, replace=False)] for u in range(2)])
    mub = narrow(widen(mub) + 0.05 * rng.standard_normal(mub.shape).astype(np.float32))
    ix = IceIndex(1, 2, 4, n, 16, C, kmeans_iters=1)
    a, best = ix.debug_assign(up(K), up(mub))
    a, best = down(a), down(best)
    for u in range(2):
        assert a[u].min() >= 0 and a[u].max() < C
        _check_assign(K[u], mub[u], a[u], "n=%d C=%d u=%d" % (n, C, u))
        _, ref_best, _ = orc.assign(K[u], mub[u])
        np.testing.assert_allclose(best[u], ref_best, rtol=0, atol=float(_assign_band(K[u], mub[u]).max()))


def test_debug_assign_exact_ties_take_lowest_id():
    from paper_2604_10539_amd import IceIndex
    rng = np.random.default_rng(3)
    n = 700
    K = narrow(rng.standard_normal((1, n, D)).astype(np.float32))
    base = narrow(rng.standard_normal((1, 40, D)).astype(np.float32))
    mub = np.concatenate([base, base], axis=1)             # centroid c+40 duplicates centroid c
    ix = IceIndex(1, 1, 4, n, 16, 80, kmeans_iters=1)
    a, _ = ix.debug_assign(up(K), up(mub))
    a = down(a)
    assert a.max() < 40
    _check_assign(K[0], base[0], a[0], "duplicates")


# ----------------------------------------------------------------------------------------- build
@pytest.mark.parametrize("kw", [
    dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32),                 # config 1 shape
    dict(n_tokens=5003, n_clusters=100, n_kv_heads=3, n_components=40),                # ragged everywhere
    dict(n_tokens=2500, n_clusters=24, n_kv_heads=2, page_size=32, n_components=12),
    dict(n_tokens=2600, n_clusters=40, n_kv_heads=1, page_size=64, group_size=8, n_components=12),
    dict(n_tokens=6000, n_clusters=600, n_kv_heads=2, n_components=200),               # two centroid slices
    dict(n_tokens=9000, n_clusters=2500, n_kv_heads=1, n_components=300),              # sort with 12 segments
    dict(n_tokens=70000, n_clusters=64, n_kv_heads=1, n_components=64),                # sort segments of 69 groups
    dict(n_tokens=9000, n_clusters=8192, n_kv_heads=1, n_components=300),             # the largest cluster count: 16 centroid slices, one sort segment
])
def test_build_stepwise_parity(kw):
    """Per-step protocol: each stage is compared with the oracle on the GPU's own previous stage."""
    T = 3
    w = datagen.small(**kw)
    ix, K, V, idx = _mk(w, T=T)
    ix.build_index(up(K), up(V))
    ex = export_np(ix)
    n, C, s = w.n_tokens, w.n_clusters, w.page_size
    assert np.array_equal(ex["init_idx"], idx)
    a_gpu = ex["assign"][:, :n]
    o = orc.OracleIndex(ix.U, w.group_size, s, C, n)
    o.paginate(K, V, a_gpu)
    for u in range(ix.U):
        # (a) last assignment against the bf16 centroids it was computed from
        _check_assign(K[u], ex["assign_centroid_bf16"][u, :C], a_gpu[u], "build u=%d" % u)
        # (b) means of the GPU's own assignment: counts exact, sums/means to fp32 accuracy
        prev = widen(ex["assign_centroid_bf16"][u, :C])
        mu, ssum, cnt = orc.means(K[u], a_gpu[u], C, prev)
        assert np.array_equal(ex["cluster_cnt"][u], cnt)
        live = cnt > 0
        np.testing.assert_allclose(ex["cluster_sum"][u], ssum, rtol=1e-5, atol=1e-4)
        np.testing.assert_allclose(ex["centroid"][u][live], mu[live], rtol=1e-5, atol=1e-5)
    # (c) page layout of the GPU's own assignment: every table and every stored bit
    assert np.array_equal(ex["n_pages"], o.n_pages)
    for name in ("page_cluster", "page_fill", "page_pos", "cluster_tail"):
        assert np.array_equal(ex[name], getattr(o, name)), name
    for u in range(ix.U):
        npg = o.n_pages[u]
        m = valid_slot_mask(o.page_fill[u, :npg], s)
        assert np.array_equal(ex["Kp"][u, :npg][m], o.Kp[u, :npg][m])
        assert np.array_equal(ex["Vp"][u, :npg][m], o.Vp[u, :npg][m])
        assert np.array_equal(ex["page_sum"][u, :npg].view(np.uint32), o.page_sum[u, :npg].view(np.uint32))
        assert np.array_equal(ex["rep"][u, :npg], o.rep[u, :npg])
    # (d) the iteration as a whole: objective close to the oracle's run from the same promoted keys
    for u in range(ix.U):
        a_o, mu_o, _, _, _ = orc.lloyd(K[u], idx[u], T)
        kf = widen(K[u]).astype(np.float64)
        j_gpu = ((kf - ex["centroid"][u].astype(np.float64)[a_gpu[u]]) ** 2).sum()
        j_orc = ((kf - mu_o.astype(np.float64)[a_o]) ** 2).sum()
        assert abs(j_gpu - j_orc) <= 5e-3 * j_orc, (j_gpu, j_orc)


def test_build_is_deterministic_and_inertia_decreases():
    w = datagen.small(n_tokens=4000, n_clusters=64, n_kv_heads=2, n_components=48)
    prev_j = None
    for T in (1, 2, 4):
        ix, K, V, idx = _mk(w, T=T)
        ix.build_index(up(K), up(V))
        ex1 = export_np(ix)
        ix.build_index(up(K), up(V))           # rebuild in place
        ex2 = export_np(ix)
        for name in STATE_FIELDS + ("assign",):
            a, b = ex1[name], ex2[name]
            if name in ("Kp", "Vp", "page_sum", "rep"):
                continue                        # stale slots of unused pages may differ; live ones checked below
            assert np.array_equal(a, b), name
        for u in range(ix.U):
            npg = ex1["n_pages"][u]
            assert np.array_equal(ex1["rep"][u, :npg], ex2["rep"][u, :npg])
            assert np.array_equal(ex1["page_sum"][u, :npg].view(np.uint32), ex2["page_sum"][u, :npg].view(np.uint32))
        kf = widen(K).astype(np.float64)
        j = sum(((kf[u] - ex1["centroid"][u].astype(np.float64)[ex1["assign"][u, :w.n_tokens]]) ** 2).sum()
                for u in range(ix.U))
        if prev_j is not None:
            assert j <= prev_j * (1 + 1e-3)
        prev_j = j


def test_build_with_seed_promotes_distinct_keys():
    w = datagen.small(n_tokens=3000, n_clusters=50, n_kv_heads=2)
    ix, K, V, _ = _mk(w, T=2, init=False, seed=1234)
    ix.build_index(up(K), up(V))
    ex = export_np(ix)
    for u in range(ix.U):
        sel = ex["init_idx"][u]
        assert len(set(sel.tolist())) == 50 and sel.min() >= 0 and sel.max() < 3000
        # same protocol as with an explicit list: oracle from the exported indices
        a_o, mu_o, _, cnt_o, _ = orc.lloyd(K[u], sel, 1)
    ix2, _, _, _ = _mk(w, T=2, init=False, seed=99)
    ix2.build_index(up(K), up(V))
    assert not np.array_equal(export_np(ix2)["init_idx"], ex["init_idx"])


# ----------------------------------------------------------------------------------------- select
def _compare_select(o, q, budget, ids, n_sel, scores=None):
    """ids/n_sel from the GPU against the oracle on identical representative bits."""
    oid, ons, osc, S_all = o.select(q, budget)
    U, P = oid.shape
    ids, n_sel = ids.reshape(U, P), n_sel.reshape(U)
    assert np.array_equal(n_sel, ons)
    ties = 0
    for u in range(U):
        k = int(ons[u])
        g = ids[u, :k]
        assert np.all(np.diff(g) > 0), "ids must be ascending and distinct"
        assert np.all(ids[u, k:] == -1)
        if np.array_equal(g, oid[u, :k]):
            continue
        only_g, only_o = np.setdiff1d(g, oid[u, :k]), np.setdiff1d(oid[u, :k], g)
        thr = np.sort(S_all[u, :o.n_pages[u]])[::-1][k - 1]
        band = SCORE_TIE * max(1.0, abs(float(thr)))
        for p in np.concatenate([only_g, only_o]):
            assert abs(float(S_all[u, p]) - float(thr)) <= band, "selection differs outside the tie band"
        ties += len(only_g)
    if scores is not None:
        scores = scores.reshape(U, P)
        for u in range(U):
            k = int(ons[u])
            np.testing.assert_allclose(scores[u, :k], S_all[u, ids[u, :k]], rtol=2e-6, atol=2e-6)
    print("[select] %d page ids differ from the oracle inside the 1e-5 tie band" % ties)
    return ties


@pytest.mark.parametrize("kw,budget", [
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 256),
    (dict(n_tokens=5003, n_clusters=100, n_kv_heads=3, n_components=40), 64),
    (dict(n_tokens=5003, n_clusters=100, n_kv_heads=3, n_components=40, group_size=1), 512),
    (dict(n_tokens=2500, n_clusters=24, n_kv_heads=2, page_size=32, group_size=2), 256),
    (dict(n_tokens=2600, n_clusters=40, n_kv_heads=1, page_size=64, group_size=8), 640),
    (dict(n_tokens=300, n_clusters=6, n_kv_heads=2), 16 * 64),           # budget covers every page
    (dict(n_tokens=20000, n_clusters=300, n_kv_heads=2, n_components=128), 16),   # one page of many
    (dict(n_tokens=20000, n_clusters=300, n_kv_heads=2, n_components=128), 16 * 48),    # threshold from histograms
    (dict(n_tokens=30000, n_clusters=500, n_kv_heads=9, n_components=200), 16 * 250),   # 250 of ~2300 pages, several workgroups per unit
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 16 * 280),      # all but a few pages
])
def test_select_and_attend_on_gpu_built_index(kw, budget):
    w = datagen.small(**kw)
    ix, K, V, _ = _mk(w, T=2)
    ix.build_index(up(K), up(V))
    q = datagen.queries(w)
    ids, n_sel, scores = ix.select(up(q), budget)
    out = ix.attend(up(q), ids, n_sel)
    ex = export_np(ix)
    o = oracle_from_export(ix, ex)
    ids_n, ns_n = down(ids), down(n_sel)
    _compare_select(o, q, budget, ids_n, ns_n, down(scores))
    # attention over the GPU's own ids
    P = ids_n.shape[-1]
    ref = o.attend(q, ids_n.reshape(ix.U, P), ns_n.reshape(ix.U))
    err = np.abs(down(out).reshape(ref.shape) - ref).max()
    print("[attend] max abs err %.3g" % err)
    assert err <= ATTN_TOL and err <= ATTN_EXPECTED
    # fused call: same ids; it attends in rank order, so the output may differ in the last bits
    ids2, ns2, out2 = ix.select_attend(up(q), budget)
    assert torch.equal(ids2, ids) and torch.equal(ns2, n_sel) and (out2 - out).abs().max().item() <= 5e-6
    # loaded tokens never exceed the budget
    for u in range(ix.U):
        sel = ids_n.reshape(ix.U, P)[u, :ns_n.reshape(ix.U)[u]]
        assert ex["page_fill"][u, sel].sum() <= budget


def test_attend_with_every_page_equals_dense_attention():
    w = datagen.small(n_tokens=1500, n_clusters=20, n_kv_heads=2)
    ix, K, V, _ = _mk(w, T=2)
    ix.build_index(up(K), up(V))
    q = datagen.queries(w)
    ids, n_sel, out = ix.select_attend(up(q), 16 * 128)
    out = down(out).reshape(ix.U, w.group_size, D)
    qf = widen(q).astype(np.float64).reshape(ix.U, w.group_size, D)
    for u in range(ix.U):
        z = qf[u] @ widen(K[u]).astype(np.float64).T / math.sqrt(D)
        p = np.exp(z - z.max(1, keepdims=True))
        ref = (p / p.sum(1, keepdims=True)) @ widen(V[u]).astype(np.float64)
        assert np.abs(out[u] - ref).max() <= ATTN_EXPECTED


def test_select_ties_and_empty_selection():
    """Identical pages tie exactly: the lowest ids win.  n_selected = 0 gives zeros."""
    from paper_2604_10539_amd import IceIndex
    rng = np.random.default_rng(5)
    key = narrow(rng.standard_normal(D).astype(np.float32))
    K = np.tile(key, (1, 1, 96, 1))
    V = narrow(rng.standard_normal((1, 1, 96, D)).astype(np.float32))
    ix = IceIndex(1, 1, 2, 96, 16, 1, kmeans_iters=1, init_idx=up(np.zeros((1, 1, 1), np.int32)))
    ix.build_index(up(K), up(V))
    q = narrow(rng.standard_normal((1, 2, D)).astype(np.float32))
    ids, n_sel, _ = ix.select(up(q), 48)
    assert down(ids).ravel().tolist() == [0, 1, 2] and int(n_sel.item()) == 3
    zero = torch.zeros_like(n_sel)
    out = ix.attend(up(q), ids, zero)
    assert torch.count_nonzero(out).item() == 0
    # order of the listed pages does not matter
    out_a = ix.attend(up(q), ids, n_sel)
    out_b = ix.attend(up(q), ids.flip(-1).contiguous(), n_sel)
    assert (out_a - out_b).abs().max().item() <= 1e-6


def test_select_many_exact_ties_uses_lowest_ids():
    """More tied candidates than the fast ranking path takes (hundreds of identical pages plus a few
    distinct ones): the radix path must still return the best pages, lowest ids first among ties."""
    from paper_2604_10539_amd import IceIndex
    rng = np.random.default_rng(9)
    n = 16 * 700
    key = narrow(rng.standard_normal(D).astype(np.float32))
    K = np.tile(key, (1, 1, n, 1))
    K[0, 0, 16 * 300:16 * 303] = narrow(3.0 * widen(key))          # three pages that beat the rest
    K[0, 0, 16 * 10:16 * 12] = narrow(-1.0 * widen(key))           # two pages that lose
    V = narrow(rng.standard_normal((1, 1, n, D)).astype(np.float32))
    ix = IceIndex(1, 1, 1, n, 16, 1, kmeans_iters=1, init_idx=up(np.zeros((1, 1, 1), np.int32)))
    ix.build_index(up(K), up(V))
    q = narrow(widen(key)[None, None, :].copy())
    ids, n_sel, scores = ix.select(up(q), 16 * 8)
    assert down(ids).ravel().tolist() == [0, 1, 2, 3, 4, 300, 301, 302]
    o = oracle_from_export(ix, export_np(ix))
    _compare_select(o, q, 16 * 8, down(ids), down(n_sel), down(scores))


# ----------------------------------------------------------------------------------------- import
def test_imported_oracle_index_select_attend():
    """An index built entirely by the oracle, imported bit for bit, must select the same pages."""
    from paper_2604_10539_amd import IceIndex
    w = datagen.small(n_tokens=3000, n_clusters=48, n_kv_heads=3, n_components=24)
    K, V = datagen.keys_values(w)
    idx = datagen.init_indices(w)
    o = orc.OracleIndex(3, w.group_size, 16, 48, 3000)
    o.build(K, V, idx, 4)
    ix = IceIndex(1, 3, w.group_size, 3000, 16, 48)
    ix.import_arrays(oracle_arrays_to_device(o), 3000)
    q = datagen.queries(w)
    ids, n_sel, scores = ix.select(up(q), 256)
    _compare_select(o, q, 256, down(ids), down(n_sel), down(scores))
    out = ix.attend(up(q), ids, n_sel)
    ref = o.attend(q, down(ids).reshape(3, -1), down(n_sel).reshape(3))
    assert np.abs(down(out).reshape(ref.shape) - ref).max() <= ATTN_EXPECTED
    ex = export_np(ix)
    for name in STATE_FIELDS:
        assert np.array_equal(ex[name], getattr(o, name)), name
    # the staged selection on the imported index (centroid roundings are recomputed at import)
    _check_hier(ix, o, q, 256, 7, *ix.select_hier(up(q), 256, 7))
    assert _check_refined(ix, o, q, 256, 48, 40, *ix.select_hier(up(q), 256, 48, n_refine=40)) == 0


# ----------------------------------------------------------------------------------------- insert
@pytest.mark.parametrize("kw,steps", [
    (dict(n_tokens=2000, n_clusters=24, n_kv_heads=2, n_components=16, drift=0.01), 300),
    (dict(n_tokens=600, n_clusters=5, n_kv_heads=3, page_size=32, n_components=4, drift=0.02), 200),
    (dict(n_tokens=6000, n_clusters=700, n_kv_heads=1, n_components=64, drift=0.01), 60),   # the scan takes two rounds of tiles per wave
])
def test_insert_replay_is_bit_exact(kw, steps):
    """The oracle starts from the exported post-build state and replays every insertion; all tables
    and the ordered-fp32 quantities must match bit for bit after every step (checked at intervals
    and at the end).  A nearest-centroid decision inside the tie band is followed and counted."""
    w = datagen.small(**kw)
    ix, K, V, _ = _mk(w, T=3, extra=steps)
    ix.build_index(up(K), up(V))
    ex = export_np(ix)
    o = oracle_from_export(ix, ex)
    stream = datagen.DecodeStream(w)
    flips = 0
    exv = ix.export()                      # device views; page tables are read back every step
    for t in range(steps):
        k, v, q = stream.next()
        ku = k.reshape(ix.U, D)
        mub = narrow(o.centroid)           # centroids as both sides see them before this insertion
        ix.insert(up(k), up(v))
        torch.cuda.synchronize()
        pos_t, pc_t = down(exv["page_pos"]), down(exv["page_cluster"])
        force = np.empty(ix.U, np.int32)
        for u in range(ix.U):
            pg = np.argwhere(pos_t[u] == w.n_tokens + t)
            assert len(pg) == 1, "the new token must sit in exactly one slot"
            c_gpu = int(pc_t[u, pg[0][0]])
            a_own, best, _ = orc.assign(ku[u][None], mub[u])
            if c_gpu != a_own[0]:          # allowed only inside the tie band; the oracle then follows
                mf = widen(mub[u, c_gpu]).astype(np.float64)
                obj = (mf ** 2).sum() - 2.0 * (widen(ku[u]).astype(np.float64) * mf).sum()
                assert obj - best[0] <= _assign_band(ku[u][None], mub[u])[0], "insert picked a non-nearest centroid"
                flips += 1
            force[u] = c_gpu
        o.insert(k, v, force=force)
        if (t % 50 == 49) or t == steps - 1:
            exg = export_np(ix)
            for name in STATE_FIELDS:
                a, b = exg[name], getattr(o, name)
                for u in range(ix.U):
                    npg = o.n_pages[u]
                    if name in ("Kp", "Vp"):
                        m = valid_slot_mask(o.page_fill[u, :npg], w.page_size)
                        assert np.array_equal(a[u, :npg][m], b[u, :npg][m]), name
                    elif name in ("page_sum", "rep"):
                        assert np.array_equal(a[u, :npg], b[u, :npg]), name
                    elif name in ("cluster_sum", "centroid"):
                        assert np.array_equal(a[u].view(np.uint32), b[u].view(np.uint32)), name
                    else:
                        assert np.array_equal(a[u], b[u]), name
    print("[insert] %d steps replayed, %d tie-band flips" % (steps, flips))
    # the grown index still selects and attends like the oracle
    k, v, q = stream.next()
    ids, n_sel, out = ix.select_attend(up(q), w.token_budget)
    _compare_select(o, q, w.token_budget, down(ids), down(n_sel))
    ref = o.attend(q, down(ids).reshape(ix.U, -1), down(n_sel).reshape(ix.U))
    assert np.abs(down(out).reshape(ref.shape) - ref).max() <= ATTN_EXPECTED


def test_insert_capacity_and_state_errors():
    from paper_2604_10539_amd import IceError, IceIndex, binding
    w = datagen.small(n_tokens=500, n_clusters=8, n_kv_heads=1)
    ix, K, V, _ = _mk(w, T=1, extra=1)
    k = up(K[:, 0])
    with pytest.raises(IceError) as e:
        ix.insert(k, k)
    assert e.value.status == binding.ICE_ERR_STATE
    ix.build_index(up(K), up(V))
    ix.insert(k, k)
    with pytest.raises(IceError) as e:
        ix.insert(k, k)
    assert e.value.status == binding.ICE_ERR_CAPACITY


@pytest.mark.gpu
def test_peak_microbenchmarks_run():
    """The two measured-peak kernels of the benchmark: they must run and leave the MFMA sums they claim."""
    import torch
    from paper_2604_10539_amd import ice_debug_peak_mfma, ice_debug_peak_read
    sink = torch.zeros(1 << 19, dtype=torch.float32, device="cuda")
    buf = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    ice_debug_peak_read(buf, buf.numel() * 4, sink)
    flops = ice_debug_peak_mfma(sink, 4)
    torch.cuda.synchronize()
    assert flops == 2048 * 4 * 4 * 4 * 32768.0
    # every wave ran 4 rounds of 4 chains: a[i] = (lane + i) & 7 (all 64 lanes' row values), b[i] = i + 1
    s = sink.cpu().numpy()
    assert np.isfinite(s).all() and (s > 0).all()
    assert np.array_equal(s[:256], s[256:512])          # every workgroup computes the same sums


# ----------------------------------------------------------------------------------------- hierarchical select
def _check_hier(ix, o, q, budget, n_probe, ids, n_sel, scores, clusters, out):
    """GPU two-stage selection against the oracle on identical index bits.  Stage 1: the kept clusters
    must be the oracle's, except for clusters within the tie band of the last kept score.  Stage 2 is
    checked against the staged definition applied to the GPU's own cluster set (so a stage-1 near-tie
    does not hide a stage-2 error), with the oracle's fp32 page scores."""
    U = ix.U
    oid, ons, osc, ocl, Sc_all = o.select_hier(q, budget, n_probe)
    _, _, _, S_all = o.select(q, budget)
    ids, n_sel, clusters = down(ids).reshape(U, -1), down(n_sel).reshape(U), down(clusters).reshape(U, n_probe)
    scores = down(scores).reshape(U, -1)
    P = ids.shape[1]
    n_keep = min(n_probe, o.C)
    ties = 0
    for u in range(U):
        g = clusters[u, :n_keep]
        assert np.all(np.diff(g) > 0) and np.all(clusters[u, n_keep:] == -1) and g.min() >= 0 and g.max() < o.C
        if not np.array_equal(g, ocl[u, :n_keep]):
            thr = np.sort(Sc_all[u])[::-1][n_keep - 1]
            band = SCORE_TIE * max(1.0, abs(float(thr)))
            for c in np.setxor1d(g, ocl[u, :n_keep]):
                assert abs(float(Sc_all[u, c]) - float(thr)) <= band, "kept clusters differ outside the tie band"
            ties += 1
        kept = set(g.tolist())
        npg = int(o.n_pages[u])
        cand = [p for p in range(npg) if int(o.page_cluster[u, p]) in kept]
        k = min(P, len(cand))
        assert n_sel[u] == k
        got = ids[u, :k]
        assert np.all(np.diff(got) > 0) and np.all(ids[u, k:] == -1)
        assert set(got.tolist()) <= set(cand)
        want = sorted(sorted(cand, key=lambda p: (-S_all[u, p], p))[:k])
        if got.tolist() != want:
            thr = sorted((S_all[u, p] for p in cand), reverse=True)[k - 1]
            band = SCORE_TIE * max(1.0, abs(float(thr)))
            for p in np.setxor1d(got, want):
                assert abs(float(S_all[u, p]) - float(thr)) <= band, "pages differ outside the tie band"
            ties += 1
        np.testing.assert_allclose(scores[u, :k], S_all[u, got], rtol=2e-6, atol=2e-6)
    print("[hier] %d near-tie differences" % ties)
    if out is not None:
        ref = o.attend(q, ids, n_sel)
        err = np.abs(down(out).reshape(ref.shape) - ref).max()
        print("[hier attend] max abs err %.3g" % err)
        assert err <= ATTN_TOL and err <= ATTN_EXPECTED
    return ties


@pytest.mark.gpu
@pytest.mark.parametrize("kw,budget,n_probe", [
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 256, 4),
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 256, 1),
    (dict(n_tokens=5003, n_clusters=100, n_kv_heads=3, n_components=40), 64, 17),
    (dict(n_tokens=5003, n_clusters=100, n_kv_heads=3, n_components=40, group_size=1), 512, 100),   # every cluster
    (dict(n_tokens=5003, n_clusters=100, n_kv_heads=3, n_components=40, group_size=2), 128, 130),   # more than exist
    (dict(n_tokens=2600, n_clusters=40, n_kv_heads=1, page_size=64, group_size=8), 640, 6),
    (dict(n_tokens=20000, n_clusters=300, n_kv_heads=2, n_components=128), 256, 70),               # more than 64 kept
    (dict(n_tokens=300, n_clusters=6, n_kv_heads=2), 16 * 64, 2),                                  # budget covers all candidates
])
def test_hier_select_and_attend(kw, budget, n_probe):
    w = datagen.small(**kw)
    ix, K, V, _ = _mk(w, T=2)
    ix.build_index(up(K), up(V))
    q = datagen.queries(w)
    ids, n_sel, scores, clusters, out = ix.select_hier(up(q), budget, n_probe)
    o = oracle_from_export(ix, export_np(ix))
    _check_hier(ix, o, q, budget, n_probe, ids, n_sel, scores, clusters, out)
    # selection alone gives the same ids
    ids2, ns2, _, cl2, none = ix.select_hier(up(q), budget, n_probe, attend=False)
    assert none is None and torch.equal(ids2, ids) and torch.equal(ns2, n_sel) and torch.equal(cl2, clusters)
    if n_probe >= w.n_clusters:   # every cluster kept: the flat scan's answer
        ids_f, ns_f, _ = ix.select(up(q), budget)
        assert torch.equal(ids_f, ids) and torch.equal(ns_f, n_sel)


@pytest.mark.gpu
def test_hier_select_after_insertions_sees_appended_pages():
    w = datagen.small(n_tokens=1500, n_clusters=12, n_kv_heads=2, n_components=8, drift=0.01)
    ix, K, V, _ = _mk(w, T=2, extra=512)
    ix.build_index(up(K), up(V))
    np0 = export_np(ix)["n_pages"].copy()
    stream = datagen.DecodeStream(w, seed=21)
    for _ in range(400):
        k, v, qq = stream.next()
        ix.insert(up(k), up(v))
    ex = export_np(ix)
    assert np.all(ex["n_pages"] > np0)
    o = oracle_from_export(ix, ex)
    for n_probe in (1, 3, 12):
        ids, n_sel, scores, clusters, out = ix.select_hier(up(qq), 16 * 40, n_probe)
        _check_hier(ix, o, qq, 16 * 40, n_probe, ids, n_sel, scores, clusters, out)
    # the best cluster's appended pages are among the winners when the budget covers the cluster
    ids, n_sel, _, clusters, _ = ix.select_hier(up(qq), 16 * 400, 1, attend=False)
    ids, n_sel, clusters = down(ids).reshape(ix.U, -1), down(n_sel).reshape(ix.U), down(clusters).reshape(ix.U, 1)
    for u in range(ix.U):
        mine = [p for p in range(ex["n_pages"][u]) if ex["page_cluster"][u, p] == clusters[u, 0]]
        assert ids[u, :n_sel[u]].tolist() == mine


@pytest.mark.gpu
def test_hier_select_many_exact_ties_takes_the_overflow_path():
    """Hundreds of identical pages in one kept cluster overflow the short ranking list: the radix
    path must return the best pages, lowest ids first among exact ties."""
    from paper_2604_10539_amd import IceIndex
    rng = np.random.default_rng(19)
    n = 16 * 700
    key = narrow(rng.standard_normal(D).astype(np.float32))
    K = np.tile(key, (1, 1, n, 1))
    K[0, 0, 16 * 300:16 * 303] = narrow(3.0 * widen(key))
    V = narrow(rng.standard_normal((1, 1, n, D)).astype(np.float32))
    ix = IceIndex(1, 1, 1, n, 16, 1, kmeans_iters=1, init_idx=up(np.zeros((1, 1, 1), np.int32)))
    ix.build_index(up(K), up(V))
    q = narrow(widen(key)[None, None, :].copy())
    ids, n_sel, scores, clusters, out = ix.select_hier(up(q), 16 * 8, 1)
    assert down(ids).ravel().tolist() == [0, 1, 2, 3, 4, 300, 301, 302]
    o = oracle_from_export(ix, export_np(ix))
    _check_hier(ix, o, q, 16 * 8, 1, ids, n_sel, scores, clusters, out)


@pytest.mark.gpu
def test_hier_select_argument_errors():
    from paper_2604_10539_amd import IceError, binding as b
    w = datagen.small(n_tokens=600, n_clusters=6, n_kv_heads=1)
    ix, K, V, _ = _mk(w, T=1)
    q = up(datagen.queries(w))
    with pytest.raises(IceError) as e:
        ix.select_hier(q, 64, 2)
    assert e.value.status == b.ICE_ERR_STATE
    ix.build_index(up(K), up(V))
    for budget, n_probe, status in ((8, 2, b.ICE_ERR_SHAPE), (64, 0, b.ICE_ERR_SHAPE)):
        with pytest.raises(IceError) as e:
            ix.select_hier(q, budget, n_probe)
        assert e.value.status == status


@pytest.mark.gpu
@pytest.mark.parametrize("kw,m,mode", [
    (dict(n_tokens=2000, n_clusters=24, n_kv_heads=2, n_components=16, drift=0.01), 16, "foreign"),
    (dict(n_tokens=600, n_clusters=3, n_kv_heads=3, page_size=32, n_components=2, drift=0.02), 32, "foreign"),   # same cluster again and again
    (dict(n_tokens=900, n_clusters=40, n_kv_heads=1, group_size=8, n_components=8), 5, "foreign"),
    (dict(n_tokens=4000, n_clusters=200, n_kv_heads=2, n_components=100, drift=0.01), 16, "own"),      # mostly one token per cluster: the guesses stand
    (dict(n_tokens=6000, n_clusters=1500, n_kv_heads=1, n_components=64), 16, "own"),                  # many clusters: fewer tokens per launch, one staging tile per wave
    (dict(n_tokens=1500, n_clusters=20, n_kv_heads=2, n_components=10), 16, "same"),                   # 16 copies of one key: one cluster, pages overflow inside a launch
    (dict(n_tokens=2500, n_clusters=64, n_kv_heads=2, n_components=32, drift=0.01), 17, "own"),         # a launch of 16 and a launch of one
    (dict(n_tokens=9000, n_clusters=4500, n_kv_heads=1, n_components=64), 6, "own"),                   # two tokens per launch; the one-token scan takes nine rounds of tiles
])
def test_insert_batch_equals_one_by_one(kw, m, mode):
    """m tokens in one launch leave the index bit for bit as m single insertions do (each token sees
    the centroid the previous one moved, pages fill and open in the same order).  foreign: the tokens
    come from other centres than the index was built on and crowd into few clusters; own: from the
    index's own stream; same: every launch repeats one key."""
    w = datagen.small(**kw)
    rounds = 4
    ix_a, K, V, _ = _mk(w, T=2, extra=rounds * m)
    ix_b, _, _, _ = _mk(w, T=2, extra=rounds * m)
    ix_a.build_index(up(K), up(V))
    ix_b.build_index(up(K), up(V))
    stream = datagen.DecodeStream(w, seed=5 if mode == "foreign" else None)
    U = ix_a.U
    for _ in range(rounds):
        ks, vs = [], []
        for j in range(m):
            k, v, _ = stream.next()
            if mode == "same" and j > 0:
                k = ks[0].reshape(k.shape).copy()
            ix_a.insert(up(k), up(v))
            ks.append(k.reshape(U, D))
            vs.append(v.reshape(U, D))
        kb = np.stack(ks, 1).reshape(w.batch, w.n_kv_heads, m, D)
        vb = np.stack(vs, 1).reshape(w.batch, w.n_kv_heads, m, D)
        ix_b.insert_batch(up(kb), up(vb))
    ea, eb = export_np(ix_a), export_np(ix_b)
    assert ea["n_tokens"] == eb["n_tokens"] == w.n_tokens + rounds * m
    assert np.array_equal(ea["n_pages"], eb["n_pages"]) and np.array_equal(ea["page_fill"], eb["page_fill"])
    for u in range(U):
        npg = int(ea["n_pages"][u])
        live = valid_slot_mask(ea["page_fill"][u, :npg], w.page_size)     # slots past the fill of a page are never written
        for name in STATE_FIELDS:
            a, b = ea[name][u], eb[name][u]
            if name in ("Kp", "Vp", "page_pos"):
                a, b = a[:npg][live], b[:npg][live]
            elif name in ("page_cluster", "page_fill", "page_sum", "rep"):
                a, b = a[:npg], b[:npg]
            assert np.array_equal(np.ascontiguousarray(a).view(np.uint8), np.ascontiguousarray(b).view(np.uint8)), name
    # and the selection on top of it is the same
    q = up(datagen.queries(w))
    ia, na, _ = ix_a.select(q, 16 * w.page_size)
    ib, nb, _ = ix_b.select(q, 16 * w.page_size)
    assert torch.equal(ia, ib) and torch.equal(na, nb)
    # capacity: one token too many is refused as a whole
    from paper_2604_10539_amd import IceError, binding as b
    with pytest.raises(IceError) as e:
        ix_b.insert_batch(up(kb[:, :, :1]), up(vb[:, :, :1]))
    assert e.value.status == b.ICE_ERR_CAPACITY


@pytest.mark.gpu
def test_insert_after_import_equals_insert_after_build():
    """What the insertions keep beside every cluster (its tail page's fill and key sum) is rebuilt from
    the page tables when an index is imported: the same tokens inserted into the built index and into
    an import of its exported state leave the same bits, one at a time and a page at a time."""
    from paper_2604_10539_amd import IceIndex
    w = datagen.small(n_tokens=3000, n_clusters=50, n_kv_heads=2, n_components=30, drift=0.01)
    extra = 48
    ix_a, K, V, _ = _mk(w, T=2, extra=extra)
    ix_a.build_index(up(K), up(V))
    ix_b = IceIndex(w.batch, w.n_kv_heads, w.group_size, w.n_tokens + extra, w.page_size, w.n_clusters, kmeans_iters=2)
    from paper_2604_10539_amd.binding import IMPORT_FIELDS
    exa = ix_a.export()
    ix_b.import_arrays({name: exa[name].clone() for name in IMPORT_FIELDS}, w.n_tokens)
    stream = datagen.DecodeStream(w)
    U = ix_a.U
    ks, vs, _ = stream.take(extra)
    for t in range(16):
        for ix in (ix_a, ix_b):
            ix.insert(up(ks[t]), up(vs[t]))
    for r in (1, 2):
        kb = up(np.ascontiguousarray(ks[16 * r:16 * r + 16].transpose(1, 2, 0, 3)))
        vb = up(np.ascontiguousarray(vs[16 * r:16 * r + 16].transpose(1, 2, 0, 3)))
        for ix in (ix_a, ix_b):
            ix.insert_batch(kb, vb)
    ea, eb = export_np(ix_a), export_np(ix_b)
    assert np.array_equal(ea["n_pages"], eb["n_pages"])
    for u in range(U):
        npg = int(ea["n_pages"][u])
        live = valid_slot_mask(ea["page_fill"][u, :npg], w.page_size)
        for name in STATE_FIELDS:
            a, b = ea[name][u], eb[name][u]
            if name in ("Kp", "Vp", "page_pos"):
                a, b = a[:npg][live], b[:npg][live]
            elif name in ("page_cluster", "page_fill", "page_sum", "rep"):
                a, b = a[:npg], b[:npg]
            assert np.array_equal(np.ascontiguousarray(a).view(np.uint8), np.ascontiguousarray(b).view(np.uint8)), name


# ----------------------------------------------------------------------------------------- resident tokens
@pytest.mark.gpu
@pytest.mark.parametrize("kw,budget,n_res", [
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 256, 37),
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 256, 1),
    (dict(n_tokens=5003, n_clusters=100, n_kv_heads=3, n_components=40, group_size=1), 64, 16),
    (dict(n_tokens=2500, n_clusters=24, n_kv_heads=2, page_size=32, group_size=2), 256, 300),
    (dict(n_tokens=2600, n_clusters=40, n_kv_heads=1, page_size=64, group_size=8), 640, 129),
])
def test_attention_with_resident_tokens(kw, budget, n_res):
    """Sink / window tokens kept by the caller as a dense run join the pages in one softmax."""
    w = datagen.small(**kw)
    ix, K, V, _ = _mk(w, T=2)
    ix.build_index(up(K), up(V))
    q = datagen.queries(w)
    rng = np.random.default_rng(n_res)
    # resident keys near the query's cluster centres so that they carry real weight
    rk = narrow((widen(K[:, :n_res]) + 0.1 * rng.standard_normal((ix.U, n_res, D))).astype(np.float32))
    rv = narrow(rng.standard_normal((ix.U, n_res, D)).astype(np.float32))
    rk4, rv4 = rk.reshape(w.batch, w.n_kv_heads, n_res, D), rv.reshape(w.batch, w.n_kv_heads, n_res, D)
    ids, n_sel, _ = ix.select(up(q), budget)
    out = ix.attend_resident(up(q), ids, n_sel, up(rk4), up(rv4))
    o = oracle_from_export(ix, export_np(ix))
    P = ids.shape[-1]
    ref = o.attend_resident(q, down(ids).reshape(ix.U, P), down(n_sel).reshape(ix.U), rk, rv)
    err = np.abs(down(out).reshape(ref.shape) - ref).max()
    plain = o.attend(q, down(ids).reshape(ix.U, P), down(n_sel).reshape(ix.U))
    print("[resident] max abs err %.3g (resident tokens move the output by %.3g)" % (err, np.abs(ref - plain).max()))
    assert err <= ATTN_TOL and err <= ATTN_EXPECTED
    assert np.abs(ref - plain).max() > 1e-3                       # the case is not vacuous
    # fused call: same ids as the plain selection, same output up to summation order
    ids2, ns2, out2 = ix.select_attend_resident(up(q), budget, up(rk4), up(rv4))
    assert torch.equal(ids2, ids) and torch.equal(ns2, n_sel) and (out2 - out).abs().max().item() <= 5e-6
    # only resident tokens
    out0 = ix.attend_resident(up(q), ids, torch.zeros_like(n_sel), up(rk4), up(rv4))
    ref0 = o.attend_resident(q, down(ids).reshape(ix.U, P), np.zeros(ix.U, np.int32), rk, rv)
    assert np.abs(down(out0).reshape(ref0.shape) - ref0).max() <= ATTN_EXPECTED
    # none: exactly the plain calls
    empty = torch.empty((w.batch, w.n_kv_heads, 0, D), dtype=torch.int16, device="cuda")
    assert torch.equal(ix.attend_resident(up(q), ids, n_sel, empty, empty), ix.attend(up(q), ids, n_sel))


# ----------------------------------------------------------------------------------------- selection reuse
@pytest.mark.gpu
@pytest.mark.parametrize("kw,budget", [
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 256),
    (dict(n_tokens=5003, n_clusters=100, n_kv_heads=3, n_components=40, group_size=1), 64),
    (dict(n_tokens=2600, n_clusters=40, n_kv_heads=1, page_size=64, group_size=8), 640),
])
def test_selection_reused_by_token_position(kw, budget):
    """An anchor layer's selection, turned into token positions, drives attention over another
    layer's dense cache; on the anchor layer's own cache it reproduces the page attention."""
    w = datagen.small(**kw)
    ix, K, V, _ = _mk(w, T=2)
    ix.build_index(up(K), up(V))
    q = datagen.queries(w)
    ids, n_sel, _ = ix.select(up(q), budget)
    pos, n_tok = ix.selected_tokens(ids, n_sel)
    o = oracle_from_export(ix, export_np(ix))
    P = ids.shape[-1]
    opos, ont = o.selected_tokens(down(ids).reshape(ix.U, P), down(n_sel).reshape(ix.U))
    assert np.array_equal(down(pos).reshape(opos.shape), opos) and np.array_equal(down(n_tok).reshape(-1), ont)
    K4, V4 = K.reshape(w.batch, w.n_kv_heads, -1, D), V.reshape(w.batch, w.n_kv_heads, -1, D)
    own = ix.attend_tokens(up(q), up(K4), up(V4), pos, n_tok)
    by_page = ix.attend(up(q), ids, n_sel)
    assert (own - by_page).abs().max().item() <= 5e-6
    rng = np.random.default_rng(budget)
    K2 = narrow((widen(K) + 0.2 * rng.standard_normal(K.shape)).astype(np.float32))
    V2 = narrow(rng.standard_normal(V.shape).astype(np.float32))
    other = ix.attend_tokens(up(q), up(K2.reshape(K4.shape)), up(V2.reshape(V4.shape)), pos, n_tok)
    ref = orc.attend_tokens(q.reshape(ix.U, w.group_size, D), K2, V2, opos, ont)
    err = np.abs(down(other).reshape(ref.shape) - ref).max()
    print("[attend by position] max abs err %.3g" % err)
    assert err <= ATTN_TOL and err <= ATTN_EXPECTED


# ----------------------------------------------------------------------------------------- random shapes
@pytest.mark.gpu
@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes_end_to_end(seed):
    """Ten random configurations per seed (page size, group size, context, clusters, heads, budget,
    probes, batched insertions, resident tokens): every decode entry point against the oracle."""
    rng = np.random.default_rng(seed)
    for case in range(10):
        s = int(rng.choice([16, 16, 32, 64]))
        G = int(rng.choice([1, 2, 4, 4, 8]))
        n = int(rng.integers(s * 4, 9000))
        C = int(rng.integers(1, min(300, n // 2)))
        H = int(rng.integers(1, 4))
        budget, n_probe = s * int(rng.integers(1, 70)), int(rng.integers(1, C + 3))
        kw = dict(n_tokens=n, n_clusters=C, n_kv_heads=H, page_size=s, group_size=G,
                  n_components=int(rng.integers(1, 64)), seed=int(rng.integers(1 << 30)))
        print("case", case, kw, "budget", budget, "n_probe", n_probe, flush=True)
        w = datagen.small(**kw)
        ix, K, V, _ = _mk(w, T=2, extra=64)
        ix.build_index(up(K), up(V))
        m = int(rng.integers(0, 40))
        if m:
            stream = datagen.DecodeStream(w, seed=case)
            toks = [stream.next()[:2] for _ in range(m)]
            kb = np.stack([k.reshape(ix.U, D) for k, _ in toks], 1).reshape(1, H, m, D)
            vb = np.stack([v.reshape(ix.U, D) for _, v in toks], 1).reshape(1, H, m, D)
            ix.insert_batch(up(kb), up(vb))
        q = datagen.queries(w)
        o = oracle_from_export(ix, export_np(ix))
        ids, n_sel, scores = ix.select(up(q), budget)
        _compare_select(o, q, budget, down(ids), down(n_sel), down(scores))
        ids2, ns2, out = ix.select_attend(up(q), budget)
        assert torch.equal(ids2, ids) and torch.equal(ns2, n_sel)
        P = ids.shape[-1]
        idn, nsn = down(ids).reshape(ix.U, P), down(n_sel).reshape(ix.U)
        assert np.abs(down(out).reshape(ix.U, G, D) - o.attend(q, idn, nsn)).max() <= ATTN_EXPECTED
        _check_hier(ix, o, q, budget, n_probe, *ix.select_hier(up(q), budget, n_probe))
        n_res = int(rng.integers(1, 200))
        rk = narrow((2 * rng.standard_normal((ix.U, n_res, D))).astype(np.float32))
        rv = narrow(rng.standard_normal((ix.U, n_res, D)).astype(np.float32))
        _, _, outr = ix.select_attend_resident(up(q), budget, up(rk.reshape(1, H, n_res, D)), up(rv.reshape(1, H, n_res, D)))
        assert np.abs(down(outr).reshape(ix.U, G, D) - o.attend_resident(q, idn, nsn, rk, rv)).max() <= ATTN_EXPECTED
        pos, n_tok = ix.selected_tokens(ids, n_sel)
        by_pos = ix.attend_tokens(up(q), up(K.reshape(1, H, n, D)), up(V.reshape(1, H, n, D)), pos, n_tok) if m == 0 else None
        if by_pos is not None:   # (without insertions every indexed token is a row of the build cache)
            assert (by_pos - ix.attend(up(q), ids, n_sel)).abs().max().item() <= 2e-5
        ix.close()


# ----------------------------------------------------------------------------------------- three levels
def _check_hier3(ix, o, q, budget, n_probe_top, n_probe, top_c, top_of, ids, n_sel, scores, clusters, tops, out):
    """GPU three-level selection against the oracle on identical index and top-level bits, stage by stage
    (each stage on the GPU's own previous stage, with the oracle's fp32 scores and the 1e-5 tie band)."""
    U = ix.U
    C2 = top_c.shape[1]
    _, _, _, _, _, Sc_all, St_all = o.select_hier3(q, budget, n_probe_top, n_probe, top_c, top_of)
    oid, ons, osc, ocl, otp, _, _ = o.select_hier3(q, budget, n_probe_top, n_probe, top_c, top_of)
    _, _, _, S_all = o.select(q, budget)
    ids, n_sel, scores = down(ids).reshape(U, -1), down(n_sel).reshape(U), down(scores).reshape(U, -1)
    clusters, tops = down(clusters).reshape(U, n_probe), down(tops).reshape(U, n_probe_top)
    P = ids.shape[1]
    ties = 0

    def same_or_tied(got, want, score_of, pool, k, what):
        if list(got) == list(want):
            return 0
        thr = sorted((score_of(x) for x in pool), reverse=True)[k - 1]
        for x in np.setxor1d(got, want):
            assert abs(float(score_of(x)) - float(thr)) <= SCORE_TIE * max(1.0, abs(float(thr))), what + " differ outside the tie band"
        return 1

    for u in range(U):
        k0 = min(n_probe_top, C2)
        g0 = tops[u, :k0]
        assert np.all(np.diff(g0) > 0) and np.all(tops[u, k0:] == -1) and g0.min() >= 0 and g0.max() < C2
        want0 = sorted(sorted(range(C2), key=lambda t: (-St_all[u, t], t))[:k0])
        ties += same_or_tied(g0, want0, lambda t: St_all[u, t], range(C2), k0, "kept top nodes")
        children = [c for c in range(o.C) if int(top_of[u, c]) in set(g0.tolist())]
        k1 = min(n_probe, len(children))
        g1 = clusters[u, :k1]
        assert np.all(np.diff(g1) > 0) and np.all(clusters[u, k1:] == -1) and set(g1.tolist()) <= set(children)
        want1 = sorted(sorted(children, key=lambda c: (-Sc_all[u, c], c))[:k1])
        if k1:
            ties += same_or_tied(g1, want1, lambda c: Sc_all[u, c], children, k1, "kept clusters")
        kept = set(g1.tolist())
        cand = [p for p in range(int(o.n_pages[u])) if int(o.page_cluster[u, p]) in kept]
        k = min(P, len(cand))
        assert n_sel[u] == k
        got = ids[u, :k]
        assert np.all(np.diff(got) > 0) and np.all(ids[u, k:] == -1) and set(got.tolist()) <= set(cand)
        want = sorted(sorted(cand, key=lambda p: (-S_all[u, p], p))[:k])
        if k:
            ties += same_or_tied(got, want, lambda p: S_all[u, p], cand, k, "pages")
        np.testing.assert_allclose(scores[u, :k], S_all[u, got], rtol=2e-6, atol=2e-6)
        if list(g0) == want0 and list(g1) == want1 and list(got) == want:   # then it IS the oracle's answer
            assert otp[u, :k0].tolist() == want0 and ocl[u, :k1].tolist() == want1 and ons[u] == k and oid[u, :k].tolist() == want
    print("[hier3] %d near-tie differences" % ties)
    if out is not None:
        ref = o.attend(q, ids, n_sel)
        assert np.abs(down(out).reshape(ref.shape) - ref).max() <= ATTN_EXPECTED
    return ties


@pytest.mark.gpu
@pytest.mark.parametrize("kw,n_top,iters", [
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 6, 1),
    (dict(n_tokens=6000, n_clusters=600, n_kv_heads=2, n_components=200), 24, 3),
    (dict(n_tokens=9000, n_clusters=2500, n_kv_heads=1, n_components=300), 256, 2),
    (dict(n_tokens=700, n_clusters=5, n_kv_heads=2), 5, 2),
])
def test_top_level_build_stepwise_parity(kw, n_top, iters):
    """The level above the clusters: promoted clusters, nearest-node assignment of the bf16 centroids,
    node means; each stage against the oracle's routines on the GPU's own previous stage."""
    w = datagen.small(**kw)
    ix, K, V, _ = _mk(w, T=2)
    ix.build_index(up(K), up(V))
    ix.build_top_level(n_top, iters)
    ex = export_np(ix)
    tl = {k2: (down(v2) if torch.is_tensor(v2) else v2) for k2, v2 in ix.export_top_level().items()}
    C = w.n_clusters
    assert tl["n_top"] == n_top
    want_init = [((2 * t + 1) * C) // (2 * n_top) for t in range(n_top)]
    for u in range(ix.U):
        pts = narrow(ex["centroid"][u])                                     # the clusters' bf16 centroids: the points
        assert tl["top_init"][u].tolist() == want_init
        top_of = tl["top_of"][u]
        assert top_of.min() >= 0 and top_of.max() < n_top
        if iters == 1:   # the only assignment was computed against the promoted rows
            _check_assign(pts, pts[want_init], top_of, "top level u=%d" % u)
        # node = mean of its clusters' points (fp32 sums in ascending cluster id); an empty node keeps its place
        mu, ssum, cnt = orc.means(pts, top_of, n_top, tl["top_centroid"][u])
        assert np.array_equal(tl["top_count"][u], cnt)
        live = cnt > 0
        np.testing.assert_allclose(tl["top_centroid"][u][live], mu[live], rtol=1e-5, atol=1e-5)
        assert np.array_equal(tl["top_centroid_bf16"][u, :n_top], narrow(tl["top_centroid"][u]))
        assert not tl["top_centroid_bf16"][u, n_top:].any()
        # the whole iteration: objective close to the oracle's run from the same promoted clusters
        a_o, mu_o, _, _, _ = orc.lloyd(pts, np.array(want_init, np.int32), iters)
        pf = widen(pts).astype(np.float64)
        j_gpu = ((pf - tl["top_centroid"][u].astype(np.float64)[top_of]) ** 2).sum()
        j_orc = ((pf - mu_o.astype(np.float64)[a_o]) ** 2).sum()
        assert abs(j_gpu - j_orc) <= 5e-3 * max(j_orc, 1e-9), (j_gpu, j_orc)
    # a rebuild of the index drops the level
    from paper_2604_10539_amd import IceError, binding as b
    ix.build_index(up(K), up(V))
    with pytest.raises(IceError) as e:
        ix.select_hier3(up(datagen.queries(w)), 64, 2, 2)
    assert e.value.status == b.ICE_ERR_STATE


@pytest.mark.gpu
@pytest.mark.parametrize("kw,budget,n_top,n_probe_top,n_probe", [
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 256, 6, 2, 8),
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 256, 6, 1, 32),
    (dict(n_tokens=5003, n_clusters=100, n_kv_heads=3, n_components=40), 64, 10, 3, 17),
    (dict(n_tokens=6000, n_clusters=600, n_kv_heads=2, n_components=200), 128, 24, 5, 60),
    (dict(n_tokens=2500, n_clusters=24, n_kv_heads=2, page_size=32, group_size=2), 256, 4, 2, 6),
    (dict(n_tokens=2600, n_clusters=40, n_kv_heads=1, page_size=64, group_size=8), 640, 8, 3, 12),
    (dict(n_tokens=9000, n_clusters=2500, n_kv_heads=1, n_components=300), 512, 256, 40, 200),
])
def test_three_level_selection_on_gpu_built_index(kw, budget, n_top, n_probe_top, n_probe):
    w = datagen.small(**kw)
    ix, K, V, _ = _mk(w, T=2, extra=40)
    ix.build_index(up(K), up(V))
    ix.build_top_level(n_top, 2)
    # insertions afterwards move centroids and open pages; the level above stays as built
    stream = datagen.DecodeStream(w, seed=9)
    for _ in range(40):
        k, v, _ = stream.next()
        ix.insert(up(k), up(v))
    tl = ix.export_top_level()
    top_c, top_of = down(tl["top_centroid"]), down(tl["top_of"])
    q = datagen.queries(w)
    o = oracle_from_export(ix, export_np(ix))
    res = ix.select_hier3(up(q), budget, n_probe_top, n_probe)
    assert _check_hier3(ix, o, q, budget, n_probe_top, n_probe, top_c, top_of, *res) == 0
    # every top node kept: exactly the two-level call
    a = ix.select_hier3(up(q), budget, n_top + 3, n_probe)
    b2 = ix.select_hier(up(q), budget, n_probe)
    assert torch.equal(a[0], b2[0]) and torch.equal(a[1], b2[1]) and torch.equal(a[2], b2[2]) and torch.equal(a[3], b2[3])
    assert torch.equal(a[5], b2[4])
    # with the best-key stage on top
    r = ix.select_hier3(up(q), budget, n_probe_top, n_probe, n_refine=2 * (budget // w.page_size))
    oid, ons, _, _, _, _, _ = o.select_hier3(q, budget, n_probe_top, n_probe, top_c, top_of, n_refine=2 * (budget // w.page_size))
    assert np.array_equal(down(r[0]).reshape(oid.shape), oid) and np.array_equal(down(r[1]).reshape(ons.shape), ons)


# ----------------------------------------------------------------------------------------- refinement by best key
def _check_refined(ix, o, q, budget, n_probe, n_refine, ids, n_sel, scores, clusters, out):
    """Stage 3 against the staged definition with the oracle's fp32 scores, on the GPU's own kept
    clusters (their own tie band is checked first, as in _check_hier).  A returned page may differ from
    the definition's only inside one of two tie bands: its representative score within 1e-5 of the
    stage-2 cut (the n_refine-th best representative score among the candidates, when there are more
    candidates than n_refine), or its best-key score within 1e-5 of the final cut (the P-th best-key
    score).  Returns the number of units with such differences."""
    U = ix.U
    oid, ons, osc, ocl, Sc_all = o.select_hier(q, budget, n_probe, n_refine)
    _, _, _, S_all = o.select(q, budget)
    ids, n_sel, scores = down(ids).reshape(U, -1), down(n_sel).reshape(U), down(scores).reshape(U, -1)
    clusters = down(clusters).reshape(U, n_probe)
    P = ids.shape[1]
    n_keep = min(n_probe, o.C)
    qf = widen(q).astype(np.float64).reshape(U, ix.group_size, D)
    ties = 0
    for u in range(U):
        g = clusters[u, :n_keep]
        if not np.array_equal(g, ocl[u, :n_keep]):
            thr = np.sort(Sc_all[u])[::-1][n_keep - 1]
            for c in np.setxor1d(g, ocl[u, :n_keep]):
                assert abs(float(Sc_all[u, c]) - float(thr)) <= SCORE_TIE * max(1.0, abs(float(thr))), "kept clusters differ outside the tie band"
            ties += 1
        kept = set(g.tolist())
        cand = sorted((p for p in range(int(o.n_pages[u])) if int(o.page_cluster[u, p]) in kept), key=lambda p: (-S_all[u, p], p))
        refine = cand[:n_refine]
        thr_stage2 = float(S_all[u, cand[n_refine - 1]]) if len(cand) > n_refine else None
        nq = np.linalg.norm(qf[u], axis=1)

        def best_key(p):
            kk = widen(o.Kp[u, p, :o.page_fill[u, p]]).astype(np.float64)
            return np.float32(((kk @ qf[u].T) / nq[None, :]).max())
        bk = {p: best_key(p) for p in refine}
        k = min(P, len(refine))
        assert n_sel[u] == k
        got = ids[u, :k]
        assert np.all(np.diff(got) > 0) and np.all(ids[u, k:] == -1) and set(got.tolist()) <= set(cand)
        np.testing.assert_allclose(scores[u, :k], [bk[p] if p in bk else best_key(p) for p in got], rtol=2e-6, atol=2e-6)
        want = sorted(sorted(refine, key=lambda p: (-bk[p], p))[:k])
        if np.array_equal(g, ocl[u, :n_keep]):   # same kept clusters: the definition's pages ARE the oracle's
            assert ons[u] == k and oid[u, :k].tolist() == want
            np.testing.assert_allclose(osc[u, :k], [bk[p] for p in want], rtol=1e-6, atol=1e-6)
        if got.tolist() == want:
            continue
        ties += 1
        thr_final = float(sorted(bk.values(), reverse=True)[k - 1])
        for p in np.setxor1d(got, want):
            near_final = abs(float(best_key(p)) - thr_final) <= SCORE_TIE * max(1.0, abs(thr_final))
            near_stage2 = thr_stage2 is not None and abs(float(S_all[u, p]) - thr_stage2) <= SCORE_TIE * max(1.0, abs(thr_stage2))
            assert near_final or near_stage2, "refined selection differs outside the two tie bands"
    print("[refine] %d units with near-tie differences" % ties)
    if out is not None:
        ref = o.attend(q, ids, n_sel)
        assert np.abs(down(out).reshape(ref.shape) - ref).max() <= ATTN_EXPECTED
    return ties


@pytest.mark.gpu
@pytest.mark.parametrize("kw,budget,n_probe,n_refine", [
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 256, 32, 64),     # flat candidates, 4x
    (dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32), 256, 6, 40),      # hierarchical candidates
    (dict(n_tokens=5003, n_clusters=100, n_kv_heads=3, n_components=40, group_size=1), 64, 100, 4),   # n_refine == P
    (dict(n_tokens=2500, n_clusters=24, n_kv_heads=2, page_size=32, group_size=2), 256, 24, 30),
    (dict(n_tokens=2600, n_clusters=40, n_kv_heads=1, page_size=64, group_size=8), 640, 40, 25),
    (dict(n_tokens=700, n_clusters=5, n_kv_heads=2), 128, 5, 5000),                        # more than exist
])
def test_selection_refined_by_best_key(kw, budget, n_probe, n_refine):
    w = datagen.small(**kw)
    ix, K, V, _ = _mk(w, T=2)
    ix.build_index(up(K), up(V))
    q = datagen.queries(w)
    ids, n_sel, scores, clusters, out = ix.select_hier(up(q), budget, n_probe, n_refine=n_refine)
    o = oracle_from_export(ix, export_np(ix))
    ties = _check_refined(ix, o, q, budget, n_probe, n_refine, ids, n_sel, scores, clusters, out)
    assert ties == 0
    with pytest.raises(Exception):
        ix.select_hier(up(q), budget, n_probe, n_refine=max(1, budget // w.page_size - 1) if budget // w.page_size > 1 else -1)


# ----------------------------------------------------------------------------------------- transformed keys
@pytest.mark.gpu
@pytest.mark.parametrize("kw", [
    dict(n_tokens=4096, n_clusters=32, n_kv_heads=2, n_components=32),
    dict(n_tokens=5003, n_clusters=100, n_kv_heads=3, n_components=40),
    dict(n_tokens=2500, n_clusters=24, n_kv_heads=2, page_size=32, n_components=12),
    dict(n_tokens=6000, n_clusters=600, n_kv_heads=2, n_components=200),               # two centroid slices
    dict(n_tokens=700, n_clusters=1, n_kv_heads=1),
])
def test_build_on_transformed_keys(kw):
    """Clustering geometry of Eq. 2: every key carries the extra coordinate sqrt(c^2 - ||k||^2).  The
    oracle clusters the (d+1)-dimensional rows; each stage is checked on the GPU's own previous stage."""
    from paper_2604_10539_amd import ICE_GEOMETRY_TRANSFORMED, IceIndex
    T = 3
    w = datagen.small(**kw)
    K, V = datagen.keys_values(w)
    # mixed norms, so that the extra coordinate matters
    U, n, C, s = w.batch * w.n_kv_heads, w.n_tokens, w.n_clusters, w.page_size
    K = K.reshape(U, n, D).copy()
    K[:, ::3] = narrow((1.7 * widen(K[:, ::3])).astype(np.float32))
    V = V.reshape(U, n, D)
    idx = datagen.init_indices(w).reshape(U, C)
    ix = IceIndex(w.batch, w.n_kv_heads, w.group_size, n, s, C, kmeans_iters=T, init_idx=up(idx.reshape(w.batch, w.n_kv_heads, C)),
                  geometry=ICE_GEOMETRY_TRANSFORMED)
    K4 = K.reshape(w.batch, w.n_kv_heads, n, D)
    ix.build_index(up(K4), up(V.reshape(K4.shape)))
    ex, geo = export_np(ix), {k: down(v) for k, v in ix.export_geometry().items()}
    # (a) the extra coordinate itself
    kf = widen(K).astype(np.float64)
    n2 = (kf ** 2).sum(-1)
    np.testing.assert_allclose(geo["radius_sq"], n2.max(-1), rtol=2e-6)
    a_gpu = widen(geo["key_extra"][:, :n]).astype(np.float64)
    want2 = np.maximum(geo["radius_sq"].astype(np.float64)[:, None] - n2, 0)
    assert np.all(np.abs(a_gpu ** 2 - want2) <= 2.0 ** -6 * want2 + 1e-5 * geo["radius_sq"].max())
    Ka = orc.augment(K, geo["key_extra"][:, :n])                       # [U, n, 129], the GPU's own coordinate
    assign = ex["assign"][:, :n]
    differ_from_raw = 0
    for u in range(U):
        # (b) last assignment against the augmented bf16 centroids it was computed from
        mub = np.concatenate([ex["assign_centroid_bf16"][u, :C], geo["assign_centroid_extra_bf16"][u, :C, None]], -1)
        _check_assign(Ka[u], mub, assign[u], "transformed build u=%d" % u)
        a_raw, _, _ = orc.assign(K[u], ex["assign_centroid_bf16"][u, :C])
        differ_from_raw += int((a_raw != assign[u]).sum())
        # (c) means of the GPU's own assignment, extra coordinate included
        mu, ssum, cnt = orc.means(Ka[u], assign[u], C, widen(mub))
        assert np.array_equal(ex["cluster_cnt"][u], cnt)
        live = cnt > 0
        np.testing.assert_allclose(ex["cluster_sum"][u], ssum[:, :D], rtol=1e-5, atol=1e-4)
        np.testing.assert_allclose(ex["centroid"][u][live], mu[live, :D], rtol=1e-5, atol=1e-5)
        np.testing.assert_allclose(geo["cluster_sum_extra"][u], ssum[:, D], rtol=1e-5, atol=1e-4)
        np.testing.assert_allclose(geo["centroid_extra"][u][live], mu[live, D], rtol=1e-5, atol=1e-5)
    if C > 1:
        assert differ_from_raw > 0, "the extra coordinate never mattered: the case is vacuous"
    # (d) the page layout is the plain one for that assignment
    o = orc.OracleIndex(U, w.group_size, s, C, n)
    o.paginate(K, V, assign)
    assert np.array_equal(ex["n_pages"], o.n_pages)
    for name in ("page_cluster", "page_fill", "page_pos", "cluster_tail"):
        assert np.array_equal(ex[name], getattr(o, name)), name
    for u in range(U):
        npg = o.n_pages[u]
        assert np.array_equal(ex["rep"][u, :npg], o.rep[u, :npg])
    # (e) the whole iteration: objective close to the oracle's run on the augmented rows
    for u in range(U):
        a_o, mu_o, _, _, _ = orc.lloyd(Ka[u], idx[u], T)
        kaf = widen(Ka[u]).astype(np.float64)
        cen = np.concatenate([ex["centroid"][u], geo["centroid_extra"][u][:, None]], -1).astype(np.float64)
        j_gpu = ((kaf - cen[assign[u]]) ** 2).sum()
        j_orc = ((kaf - mu_o.astype(np.float64)[a_o]) ** 2).sum()
        assert abs(j_gpu - j_orc) <= 5e-3 * j_orc, (j_gpu, j_orc)
    # selection and attention work on it as on any index
    q = datagen.queries(w)
    ids, n_sel, scores = ix.select(up(q), 128)
    _compare_select(oracle_from_export(ix, ex), q, 128, down(ids), down(n_sel), down(scores))
    # a raw rebuild of the same object gives back the raw clustering
    from paper_2604_10539_amd import ICE_GEOMETRY_RAW, ice_set_geometry
    ice_set_geometry(ix.handle, ICE_GEOMETRY_RAW)
    ix.build_index(up(K4), up(V.reshape(K4.shape)))
    assert ix.export_geometry() is None
    ex2 = export_np(ix)
    for u in range(U):
        _check_assign(K[u], ex2["assign_centroid_bf16"][u, :C], ex2["assign"][u, :n], "raw rebuild u=%d" % u)


def _oracle_with_geometry(ix, n_prefill):
    """An OracleIndex holding the bits of a GPU index built on transformed keys, geometry included."""
    ex = export_np(ix)
    geo = {a: down(b).copy() for a, b in ix.export_geometry().items()}
    o = oracle_from_export(ix, ex)
    o.set_geometry(geo["radius_sq"], geo["key_extra"], geo["centroid_extra"], geo["cluster_sum_extra"])
    return o


def _compare_state_bits(ix, o, s, geometry=False):
    exg = export_np(ix)
    for name in STATE_FIELDS:
        a, b = exg[name], getattr(o, name)
        for u in range(ix.U):
            npg = o.n_pages[u]
            if name in ("Kp", "Vp"):
                m = valid_slot_mask(o.page_fill[u, :npg], s)
                assert np.array_equal(a[u, :npg][m], b[u, :npg][m]), name
            elif name in ("page_sum", "rep"):
                assert np.array_equal(a[u, :npg], b[u, :npg]), name
            elif name in ("cluster_sum", "centroid"):
                assert np.array_equal(a[u].view(np.uint32), b[u].view(np.uint32)), name
            else:
                assert np.array_equal(a[u], b[u]), name
    if geometry:
        g = {a: down(b) for a, b in ix.export_geometry().items()}
        nt = int(o.n_tokens[0])
        assert np.array_equal(g["key_extra"][:, :nt], o.geometry["key_extra"][:, :nt]), "key_extra"
        for name in ("centroid_extra", "cluster_sum_extra", "radius_sq"):
            assert np.array_equal(g[name].view(np.uint32), o.geometry[name].view(np.uint32)), name


@pytest.mark.gpu
def test_insert_on_transformed_keys():
    """Insertion with the extra coordinate (Sec. 4.2 last paragraph, Eq. 2) against the oracle's
    insertion on transformed keys: the oracle starts from the exported post-build state and replays
    every step.  The new key's coordinate must be the oracle's, or its bf16 neighbour when the fp32 norm
    lands across a rounding boundary (counted; the oracle then follows); the chosen cluster must be the
    oracle's nearest augmented centroid or lie inside the fp32 band (counted, followed); every table and
    every ordered-fp32 quantity, extra coordinate included, must then match bit for bit.  A key longer
    than the radius gets coordinate 0."""
    from paper_2604_10539_amd import ICE_GEOMETRY_TRANSFORMED, IceIndex
    w = datagen.small(n_tokens=1500, n_clusters=12, n_kv_heads=2, n_components=8, drift=0.01)
    K, V = datagen.keys_values(w)
    U, n, C = 2, w.n_tokens, w.n_clusters
    K = K.reshape(U, n, D).copy()
    K[:, ::3] = narrow((1.7 * widen(K[:, ::3])).astype(np.float32))
    idx = datagen.init_indices(w)
    steps = 200
    ix = IceIndex(1, 2, w.group_size, n + steps, 16, C, kmeans_iters=2, init_idx=up(idx), geometry=ICE_GEOMETRY_TRANSFORMED)
    ix.build_index(up(K.reshape(1, 2, n, D)), up(V))
    o = _oracle_with_geometry(ix, n)
    stream = datagen.DecodeStream(w, seed=4)
    exv, gv = ix.export(), ix.export_geometry()
    flips = coord_flips = differs_from_raw = 0
    for step in range(steps):
        k, v, _ = stream.next()
        k = k.reshape(U, D).copy()
        if step % 3 == 1:
            k = narrow((1.7 * widen(k)).astype(np.float32))           # mixed norms among the new keys as well
        if step == 5:
            k = narrow((6.0 * widen(k)).astype(np.float32))           # longer than every prefill key
        mub = np.concatenate([narrow(o.centroid), narrow(o.geometry["centroid_extra"])[..., None]], -1)
        ix.insert(up(k.reshape(1, 2, D)), up(v))
        torch.cuda.synchronize()
        tok = n + step
        a_gpu = down(gv["key_extra"])[:, tok].copy()
        pos_t, pc_t = down(exv["page_pos"]), down(exv["page_cluster"])
        force = np.empty(U, np.int32)
        for u in range(U):
            pg = np.argwhere(pos_t[u] == tok)
            assert len(pg) == 1, "the new token must sit in exactly one slot"
            c_gpu = int(pc_t[u, pg[0][0]])
            ka = np.concatenate([k[u], a_gpu[u:u + 1]]).astype(np.uint16)[None]
            a_own, best, _ = orc.assign(ka, mub[u])
            if c_gpu != a_own[0]:
                mf = widen(mub[u, c_gpu]).astype(np.float64)
                obj = (mf ** 2).sum() - 2.0 * (widen(ka[0]).astype(np.float64) * mf).sum()
                assert obj - best[0] <= _assign_band(ka, mub[u])[0], "insert picked a non-nearest augmented centroid"
                flips += 1
            a_raw, _, _ = orc.assign(k[u][None], mub[u, :, :D].copy())
            differs_from_raw += int(a_raw[0] != c_gpu)
            force[u] = c_gpu
        _, _, _, own = o.insert(k, v, force=force, extra_override=a_gpu.astype(np.int32))
        for u in range(U):
            if own[u] != a_gpu[u]:      # neighbouring bf16 values only, and only next to a rounding boundary
                n2 = (widen(k[u]).astype(np.float64) ** 2).sum()
                c2 = float(o.geometry["radius_sq"][u])
                exact = math.sqrt(max(c2 - n2, 0.0))
                lo, hi = sorted((float(widen(own[u:u + 1])[0]), float(widen(a_gpu[u:u + 1])[0])))
                assert abs(int(own[u]) - int(a_gpu[u])) == 1, "extra coordinate is not the oracle's nor its neighbour"
                # the fp32 sum of squares and c^2 - ||k||^2 carry ~ (d+2) 2^-24 (c^2 + ||k||^2) of error
                slack = (D + 2) * U2 * (c2 + n2) / max(2.0 * exact, 1e-30)
                assert abs(exact - 0.5 * (lo + hi)) <= slack, "extra coordinate rounded away from a boundary"
                coord_flips += 1
        if step == 5:
            assert np.all(a_gpu == 0)
        if step % 20 == 19 or step == steps - 1 or step == 5:
            _compare_state_bits(ix, o, 16, geometry=True)
    print("[transformed insert] %d steps, %d cluster tie flips, %d coordinate rounding flips, %d decisions differ from raw"
          % (steps, flips, coord_flips, differs_from_raw))
    assert differs_from_raw > 0, "the extra coordinate never mattered: the case is vacuous"
    assert flips <= 2 and coord_flips <= 4
    # a page of tokens at once gives the same state as one by one
    ix_a = IceIndex(1, 2, w.group_size, n + 16, 16, C, kmeans_iters=2, init_idx=up(idx), geometry=ICE_GEOMETRY_TRANSFORMED)
    ix_b = IceIndex(1, 2, w.group_size, n + 16, 16, C, kmeans_iters=2, init_idx=up(idx), geometry=ICE_GEOMETRY_TRANSFORMED)
    for x in (ix_a, ix_b):
        x.build_index(up(K.reshape(1, 2, n, D)), up(V))
    toks = [stream.next()[:2] for _ in range(16)]
    for kk, vv in toks:
        ix_a.insert(up(kk), up(vv))
    ix_b.insert_batch(up(np.stack([kk.reshape(U, D) for kk, _ in toks], 1).reshape(1, 2, 16, D)),
                      up(np.stack([vv.reshape(U, D) for _, vv in toks], 1).reshape(1, 2, 16, D)))
    ga, gb = ix_a.export_geometry(), ix_b.export_geometry()
    for name in ("key_extra", "centroid_extra", "cluster_sum_extra", "radius_sq"):
        assert torch.equal(ga[name], gb[name]), name
    ea, eb = export_np(ix_a), export_np(ix_b)
    for name in ("cluster_cnt", "cluster_sum", "centroid", "cluster_tail", "n_pages", "page_fill"):
        assert np.array_equal(ea[name], eb[name]), name


# ------------------------------------------------------------------------------------ failure path of the score hand-off
def test_expired_score_handoff_is_reported_not_ranked():
    """Few units: a unit's page scores cross from several workgroups to the last of them through device
    memory, and that one waits for a missing score only a bounded number of re-reads.  The wait is made
    to expire from the host (one workgroup's score stores left out, a 16-re-read limit; every wave still
    runs to its end): the unit must come back as n_selected = -1 with ids -1 and a zero output, stay so
    on later calls, and work again, equal to the oracle, after a rebuild."""
    from paper_2604_10539_amd import IceError, binding as b
    w = datagen.small(n_tokens=9000, n_clusters=100, n_kv_heads=2, n_components=40)
    ix, K, V, _ = _mk(w, T=2)
    ix.build_index(up(K), up(V))
    q = datagen.queries(w)
    ids_ok, ns_ok, out_ok = ix.select_attend(up(q), 256)
    P = ids_ok.shape[-1]
    ids = torch.full_like(ids_ok, 5)
    ns = torch.full_like(ns_ok, 5)
    out = torch.full_like(out_ok, 5.0)
    b.ice_debug_select_fault(ix.handle, up(q), 256, ids, ns, out, 1, 4)
    torch.cuda.synchronize()
    assert torch.all(ns == -1) and torch.all(ids == -1) and torch.count_nonzero(out).item() == 0
    # the unit stays marked: the plain calls say so as well, and attention over "-1 pages" is zero
    ids2, ns2, out2 = ix.select_attend(up(q), 256)
    ids3, ns3, _ = ix.select(up(q), 256)
    torch.cuda.synchronize()
    assert torch.all(ns2 == -1) and torch.all(ids2 == -1) and torch.count_nonzero(out2).item() == 0
    assert torch.all(ns3 == -1) and torch.all(ids3 == -1)
    assert torch.count_nonzero(ix.attend(up(q), ids2, ns2)).item() == 0
    # argument errors of the hook
    with pytest.raises(IceError) as e:
        b.ice_debug_select_fault(ix.handle, up(q), 256, ids, ns, out, 99, 4)
    assert e.value.status == b.ICE_ERR_SHAPE
    with pytest.raises(IceError) as e:
        b.ice_debug_select_fault(ix.handle, up(q), 256, ids, ns, out, 0, 21)
    assert e.value.status == b.ICE_ERR_SHAPE
    # a rebuild re-arms the unit
    ix.build_index(up(K), up(V))
    ids4, ns4, out4 = ix.select_attend(up(q), 256)
    assert torch.equal(ids4, ids_ok) and torch.equal(ns4, ns_ok) and torch.equal(out4, out_ok)
    o = oracle_from_export(ix, export_np(ix))
    _compare_select(o, q, 256, down(ids4), down(ns4))
    ref = o.attend(q, down(ids4).reshape(ix.U, P), down(ns4).reshape(ix.U))
    assert np.abs(down(out4).reshape(ref.shape) - ref).max() <= ATTN_EXPECTED
    # one workgroup per unit: nothing is handed over, the hook says so
    w1 = datagen.small(n_tokens=700, n_clusters=16, n_kv_heads=2, n_components=8)
    ix1, K1, V1, _ = _mk(w1, T=1)
    ix1.build_index(up(K1), up(V1))
    i1, n1, o1 = ix1.select_attend(up(datagen.queries(w1)), 64)
    with pytest.raises(IceError) as e:
        b.ice_debug_select_fault(ix1.handle, up(datagen.queries(w1)), 64, i1, n1, o1, 0, 4)
    assert e.value.status == b.ICE_ERR_UNSUPPORTED


def test_rerunning_a_build_stage_leaves_the_index_as_it_was():
    """ice_debug_rerun_stage (what the benchmark times kernel by kernel) reproduces what the build wrote."""
    from paper_2604_10539_amd import IceError, binding as b
    for kw in (dict(n_tokens=6000, n_clusters=600, n_kv_heads=2, n_components=200), dict(n_tokens=3000, n_clusters=48, n_kv_heads=3)):
        w = datagen.small(**kw)
        ix, K, V, _ = _mk(w, T=3, extra=4)
        Kd, Vd = up(K), up(V)
        ix.build_index(Kd, Vd)
        before = {k2: (v2.copy() if isinstance(v2, np.ndarray) else v2) for k2, v2 in export_np(ix).items()}
        for stage in (b.ICE_STAGE_ASSIGN, b.ICE_STAGE_SORT, b.ICE_STAGE_MEANS, b.ICE_STAGE_PAGINATE, b.ICE_STAGE_ASSIGN):
            b.ice_debug_rerun_stage(ix.handle, Kd, Vd, stage)
        after = export_np(ix)
        for name, a in before.items():
            if isinstance(a, np.ndarray):
                assert np.array_equal(a.view(np.uint8), after[name].view(np.uint8)), name
        with pytest.raises(IceError) as e:
            b.ice_debug_rerun_stage(ix.handle, Kd, Vd, 7)
        assert e.value.status == b.ICE_ERR_INVALID_ARG
        ix.insert(up(K[:, 0]), up(V[:, 0]))
        with pytest.raises(IceError) as e:
            b.ice_debug_rerun_stage(ix.handle, Kd, Vd, b.ICE_STAGE_MEANS)
        assert e.value.status == b.ICE_ERR_STATE


# ------------------------------------------------------------------------------------ HIP graphs
@pytest.mark.parametrize("kw", [
    dict(n_tokens=3000, n_clusters=48, n_kv_heads=3, n_components=24),     # few units: several workgroups per unit
    dict(n_tokens=700, n_clusters=16, n_kv_heads=2, n_components=8),       # one workgroup per unit
])
def test_hip_graph_replays_match_eager_calls(kw):
    """The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no
    memset), so build and decode calls can be captured into a HIP graph.  Every replay, with eager
    work of the same kind in between, must reproduce the eager results bit for bit."""
    w = datagen.small(**kw)
    ix, K, V, _ = _mk(w, T=2)
    Kd, Vd = up(K), up(V)
    ix.build_index(Kd, Vd)
    q = up(datagen.queries(w))
    q_other = up(datagen.queries(w, step=1))
    ids_e, ns_e, out_e = ix.select_attend(q, 256)
    hid_e, hns_e, hsc_e, hcl_e, hout_e = ix.select_hier(q, 256, n_probe=8)
    state_e = export_np(ix)
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ix.select_attend(q, 256)  # (warm-up on the capture stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    g_build, g_step = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_build):
        ix.build_index(Kd, Vd)
    with torch.cuda.graph(g_step):
        ids_g, ns_g, out_g = ix.select_attend(q, 256)
        hid_g, hns_g, hsc_g, hcl_g, hout_g = ix.select_hier(q, 256, n_probe=8)
    for replay in range(3):
        # eager work between the replays: another query, and the outputs of the graph overwritten
        ix.select_attend(q_other, 256)
        out_g.fill_(7.0)
        ids_g.fill_(-5)
        hout_g.fill_(7.0)
        torch.cuda.synchronize()
        if replay == 1:
            g_build.replay()  # the same prefill again: the same index
        g_step.replay()
        torch.cuda.synchronize()
        assert torch.equal(ids_g, ids_e) and torch.equal(ns_g, ns_e), "replay %d: page ids" % replay
        assert torch.equal(out_g, out_e), "replay %d: attention output" % replay
        assert torch.equal(hid_g, hid_e) and torch.equal(hns_g, hns_e) and torch.equal(hcl_g, hcl_e)
        assert torch.equal(hsc_g, hsc_e) and torch.equal(hout_g, hout_e), "replay %d: hierarchical step" % replay
    state_g = export_np(ix)
    for name in STATE_FIELDS:
        a, b = state_e[name], state_g[name]
        for u in range(ix.U):
            npg = int(state_e["n_pages"][u])
            if name in ("Kp", "Vp"):
                m = valid_slot_mask(state_e["page_fill"][u, :npg], w.page_size)
                assert np.array_equal(a[u, :npg][m], b[u, :npg][m]), name
            elif name in ("page_sum", "rep"):
                assert np.array_equal(a[u, :npg], b[u, :npg]), name
            elif name in ("cluster_sum", "centroid"):
                assert np.array_equal(a[u].view(np.uint32), b[u].view(np.uint32)), name
            elif name == "n_pages":
                assert a[u] == b[u], name
            elif name in ("page_cluster", "page_fill", "page_pos"):
                assert np.array_equal(a[u, :npg], b[u, :npg]), name
            else:
                assert np.array_equal(a[u], b[u]), name
