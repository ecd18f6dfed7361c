"""GPU parity at the benchmark's full sizes and launch shapes.  What the oracle can compute in full
(selection over every page of every unit, attention over the selected pages) is compared in full;
what it cannot in seconds (the n x C assignment, the page layout of 256 units) is compared on
sampled keys and sampled units, plus invariants that hold at any size."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import datagen
from datagen import bf16_bits_to_f32 as widen, f32_to_bf16_bits as narrow
from oracle import ice_oracle as orc
from tests.test_gpu_parity import ATTN_EXPECTED, ATTN_TOL, _assign_band, _check_hier, _compare_select
from tests.util import D, down, up, valid_slot_mask

pytestmark = pytest.mark.gpu


def _select_attend_vs_oracle(ix, ex, q_np, budget, ids, n_sel, out):
    """Selection over all pages of all units, attention over the GPU's ids, both against the oracle.
    The oracle gets the representatives in full and only the selected K/V tiles (gathered on the GPU)."""
    U, G, s = ix.U, ix.group_size, ix.page_size
    P = ids.shape[-1]
    ids2, ns = ids.reshape(U, P), n_sel.reshape(U)
    o = orc.OracleIndex(U, G, s, ix.n_clusters, ix.max_tokens, alloc_kv=False)
    o.rep[...] = down(ex["rep"])
    o.n_pages[...] = down(ex["n_pages"])
    o.page_fill[...] = down(ex["page_fill"])
    _compare_select(o, q_np, budget, down(ids2), down(ns))
    _attend_vs_oracle(ix, ex, q_np, budget, ids, n_sel, out)


def _attend_vs_oracle(ix, ex, q_np, budget, ids, n_sel, out):
    """Attention over the GPU's ids against the oracle, which gets only the selected K/V tiles
    (gathered on the GPU) as a compact index: page j of unit u = the j-th selected page."""
    U, G, s = ix.U, ix.group_size, ix.page_size
    P = ids.shape[-1]
    ids2, ns = ids.reshape(U, P), n_sel.reshape(U)
    gi = ids2.clamp(min=0).long()
    g = orc.OracleIndex(U, G, s, ix.n_clusters, ix.max_tokens, max_pages=P)
    g.Kp[...] = down(torch.gather(ex["Kp"], 1, gi[:, :, None, None].expand(U, P, s, D)))
    g.Vp[...] = down(torch.gather(ex["Vp"], 1, gi[:, :, None, None].expand(U, P, s, D)))
    g.page_fill[...] = down(torch.gather(ex["page_fill"], 1, gi))
    g.n_pages[...] = down(ns)
    ref = g.attend(q_np, np.tile(np.arange(P, dtype=np.int32), (U, 1)), down(ns))
    err = np.abs(down(out).reshape(ref.shape) - ref).max()
    print("[full size] attention max abs err %.3g over %d units" % (err, U))
    assert err <= ATTN_TOL and err <= ATTN_EXPECTED
    fill = down(ex["page_fill"])
    for u in range(U):
        assert fill[u, down(ids2)[u, :down(ns)[u]]].sum() <= budget


def _hier_vs_oracle(ix, ex, q_np, budget, n_probe):
    """Two-stage selection + attention in one launch against the oracle (representatives, page ->
    cluster table and centroids in full; K/V only for the selected pages)."""
    ids, n_sel, scores, clusters, out = ix.select_hier(up(q_np), budget, n_probe)
    torch.cuda.synchronize()
    o = orc.OracleIndex(ix.U, ix.group_size, ix.page_size, ix.n_clusters, ix.max_tokens, alloc_kv=False)
    for name in ("rep", "n_pages", "page_fill", "page_cluster", "centroid"):
        getattr(o, name)[...] = down(ex[name])
    _check_hier(ix, o, q_np, budget, n_probe, ids, n_sel, scores, clusters, None)
    _attend_vs_oracle(ix, ex, q_np, budget, ids, n_sel, out)


def _check_units(ix, ex, K, V, units, n, rng, n_keys=256):
    """Sampled units: table invariants, bit copies, ordered-fp32 representatives (oracle page layout
    of the GPU's assignment), and the assignment itself on sampled keys."""
    s, C = ix.page_size, ix.n_clusters
    for u in units:
        a = down(ex["assign"][u, :n])
        Ku, Vu = K[u], V[u]
        o = orc.OracleIndex(1, ix.group_size, s, C, n)
        o.paginate(Ku[None], Vu[None], a[None])
        npg = int(o.n_pages[0])
        assert int(ex["n_pages"][u]) == npg
        for name in ("page_cluster", "page_fill", "cluster_tail"):
            assert np.array_equal(down(ex[name][u])[:getattr(o, name).shape[1]], getattr(o, name)[0]), name
        assert np.array_equal(down(ex["page_pos"][u, :npg]), o.page_pos[0, :npg])
        m = valid_slot_mask(o.page_fill[0, :npg], s)
        assert np.array_equal(down(ex["Kp"][u, :npg])[m], o.Kp[0, :npg][m])
        assert np.array_equal(down(ex["Vp"][u, :npg])[m], o.Vp[0, :npg][m])
        assert np.array_equal(down(ex["rep"][u, :npg]), o.rep[0, :npg])
        assert np.array_equal(down(ex["page_sum"][u, :npg]).view(np.uint32), o.page_sum[0, :npg].view(np.uint32))
        pos = o.page_pos[0, :npg][m]
        assert np.array_equal(np.sort(pos), np.arange(n))                       # every token exactly once
        # assignment on sampled keys against the centroids it was computed from
        mub = down(ex["assign_centroid_bf16"][u, :C])
        pick = rng.choice(n, n_keys, replace=False)
        a_ref, best, _ = orc.assign(Ku[pick], mub)
        kf, mf = widen(Ku[pick]).astype(np.float64), widen(mub).astype(np.float64)
        obj = (mf[a[pick]] ** 2).sum(1) - 2.0 * (kf * mf[a[pick]]).sum(1)
        assert np.all(obj - best <= _assign_band(Ku[pick], mub))
        assert (a[pick] != a_ref).sum() <= 2
        # centroids are the means of their members
        cnt = np.bincount(a, minlength=C)
        assert np.array_equal(down(ex["cluster_cnt"][u]), cnt)
        c0 = int(np.argmax(cnt))
        mean = widen(Ku[a == c0]).astype(np.float64).mean(0)
        np.testing.assert_allclose(down(ex["centroid"][u, c0]), mean, rtol=1e-5, atol=1e-5)


def test_config2_all_32_layers_in_the_bench_launch_shape():
    """256 units (32 layers x 8 KV heads), n = 32768, C = 512, budget 256: exactly what bench.py times."""
    from paper_2604_10539_amd import IceIndex
    w = datagen.WORKLOADS["cfg2"]
    L = 32

    def gen(l):
        K, V = datagen.keys_values(w, seed=w.seed + l)
        return K[0], V[0], datagen.init_indices(w, seed=w.seed + l)[0], datagen.queries(w, seed=w.seed + l)[0]

    with ThreadPoolExecutor(max_workers=16) as ex_:
        layers = list(ex_.map(gen, range(L)))
    K = np.stack([x[0] for x in layers]).reshape(L * 8, w.n_tokens, D)
    V = np.stack([x[1] for x in layers]).reshape(L * 8, w.n_tokens, D)
    init = np.stack([x[2] for x in layers])
    q_np = np.stack([x[3] for x in layers])
    del layers
    ix = IceIndex(L, 8, 4, w.n_tokens + 64, 16, 512, kmeans_iters=2, init_idx=up(init))
    ix.build_index(up(K), up(V))
    ids, n_sel, out = ix.select_attend(up(q_np), 256)
    torch.cuda.synchronize()
    ex = ix.export()
    _select_attend_vs_oracle(ix, ex, q_np, 256, ids, n_sel, out)
    _check_units(ix, ex, K, V, [0, 97, 255], w.n_tokens, np.random.default_rng(0))
    _hier_vs_oracle(ix, ex, q_np, 256, 64)                   # the benchmark's hierarchical variant
    # one layer at a time (8 units, several workgroups per unit) gives the same ids and output bits
    one = IceIndex(1, 8, 4, w.n_tokens + 64, 16, 512, kmeans_iters=2, init_idx=up(init[5]))
    one.build_index(up(K[40:48]), up(V[40:48]))
    ids1, ns1, out1 = one.select_attend(up(q_np[5:6]), 256)
    assert torch.equal(ids1[0], ids[5]) and torch.equal(out1[0], out[5])


def test_config3_shape_long_context():
    """Config 3 as the benchmark times it: all 8 KV heads, n = 131072, C = 2048 (four centroid slices),
    budget 1024 (P = 64), 5 % outlier keys: 8 units x 32 workgroups, attention split into shares."""
    from paper_2604_10539_amd import IceIndex
    w = datagen.WORKLOADS["cfg3"]
    K, V = datagen.keys_values(w)
    K, V = K.reshape(8, w.n_tokens, D), V.reshape(8, w.n_tokens, D)
    init, q_np = datagen.init_indices(w), datagen.queries(w)
    ix = IceIndex(1, 8, 4, w.n_tokens, 16, w.n_clusters, kmeans_iters=2, init_idx=up(init))
    ix.build_index(up(K), up(V))
    ids, n_sel, out = ix.select_attend(up(q_np), w.token_budget)
    torch.cuda.synchronize()
    ex = ix.export()
    _select_attend_vs_oracle(ix, ex, q_np, w.token_budget, ids, n_sel, out)
    _check_units(ix, ex, K, V, [1, 6], w.n_tokens, np.random.default_rng(1), n_keys=64)
    _hier_vs_oracle(ix, ex, q_np, w.token_budget, 256)
    # the separate calls give the same pages and the same output (other summation order)
    ids_s, ns_s, _ = ix.select(up(q_np), w.token_budget)
    assert torch.equal(ids_s, ids) and torch.equal(ns_s, n_sel)
    assert (ix.attend(up(q_np), ids, n_sel) - out).abs().max().item() <= 5e-6


def test_config4_shape_batched_sequences():
    """Config 4 in full: 16 sequences x 8 KV heads = 128 units at context 32768, C = 512, budget 256, in
    one launch (two workgroups per unit over up to 2560 pages).  Selection and attention are compared
    for every unit; page layout and assignment on sampled units."""
    from paper_2604_10539_amd import IceIndex
    w = datagen.WORKLOADS["cfg4"]
    K, V = datagen.keys_values(w)
    K, V = K.reshape(128, w.n_tokens, D), V.reshape(128, w.n_tokens, D)
    init, q_np = datagen.init_indices(w), datagen.queries(w)
    ix = IceIndex(16, 8, 4, w.n_tokens, 16, w.n_clusters, kmeans_iters=2, init_idx=up(init))
    ix.build_index(up(K), up(V))
    ids, n_sel, out = ix.select_attend(up(q_np), w.token_budget)
    torch.cuda.synchronize()
    ex = ix.export()
    _select_attend_vs_oracle(ix, ex, q_np, w.token_budget, ids, n_sel, out)
    _check_units(ix, ex, K, V, [0, 63, 127], w.n_tokens, np.random.default_rng(2))
    _hier_vs_oracle(ix, ex, q_np, w.token_budget, 64)


def test_config5_long_generation_loop():
    """Config 5 in full: prompt of 16384 tokens, then 4096 decode steps of insert -> select(256) ->
    attend with drifting centres.  The oracle replays every insertion from the exported post-build
    state; tables and ordered-fp32 state are compared bit for bit every 256 steps and at the end,
    selection and attention every 64 steps."""
    from paper_2604_10539_amd import IceIndex
    from tests.util import STATE_FIELDS, export_np, oracle_from_export
    w = datagen.WORKLOADS["cfg5"]
    steps = w.decode_steps
    K, V = datagen.keys_values(w)
    init = datagen.init_indices(w)
    ix = IceIndex(1, 8, 4, w.n_tokens + steps, 16, w.n_clusters, kmeans_iters=3, init_idx=up(init))
    ix.build_index(up(K), up(V))
    o = oracle_from_export(ix, export_np(ix))
    exv = ix.export()
    stream = datagen.DecodeStream(w)
    flips = 0
    pages0 = o.n_pages.copy()

    def compare_state():
        exg = export_np(ix)
        for name in STATE_FIELDS:
            a, b = exg[name], getattr(o, name)
            for u in range(8):
                npg = o.n_pages[u]
                if name in ("Kp", "Vp"):
                    m = valid_slot_mask(o.page_fill[u, :npg], 16)
                    assert np.array_equal(a[u, :npg][m], b[u, :npg][m]), name
                elif name in ("page_sum", "rep"):
                    assert np.array_equal(a[u, :npg], b[u, :npg]), name
                elif name in ("cluster_sum", "centroid"):
                    assert np.array_equal(a[u].view(np.uint32), b[u].view(np.uint32)), name
                else:
                    assert np.array_equal(a[u], b[u]), name

    for t in range(steps):
        k, v, q = stream.next()
        ku = k.reshape(8, D)
        mub = narrow(o.centroid)
        ix.insert(up(k), up(v))
        ids, n_sel, out = ix.select_attend(up(q), 256)
        torch.cuda.synchronize()
        pos_t, pc_t = down(exv["page_pos"]), down(exv["page_cluster"])
        force = np.empty(8, np.int32)
        for u in range(8):
            pg = np.argwhere(pos_t[u] == w.n_tokens + t)
            assert len(pg) == 1
            force[u] = pc_t[u, pg[0][0]]
            a_own, best, _ = orc.assign(ku[u][None], mub[u])
            if force[u] != a_own[0]:
                mf = widen(mub[u, force[u]]).astype(np.float64)
                obj = (mf ** 2).sum() - 2.0 * (widen(ku[u]).astype(np.float64) * mf).sum()
                assert obj - best[0] <= _assign_band(ku[u][None], mub[u])[0]
                flips += 1
        o.insert(k, v, force=force)
        if t % 64 == 63 or t == steps - 1:
            _compare_select(o, q, 256, down(ids), down(n_sel))
            ref = o.attend(q, down(ids).reshape(8, -1), down(n_sel).reshape(8))
            assert np.abs(down(out).reshape(ref.shape) - ref).max() <= ATTN_EXPECTED
        if t % 256 == 255 or t == steps - 1:
            compare_state()
            print("[config 5] step %d: state equal, %d pages opened so far" % (t + 1, int((o.n_pages - pages0).sum())), flush=True)
    assert flips <= steps * 8 // 500
    print("[config 5] %d steps, %d nearest-centroid decisions inside the tie band" % (steps, flips))


def test_context_of_300k_tokens_on_the_flat_path():
    """The paper's longest latency point (300k tokens): 20 798 pages per unit at page size 16, more than one
    workgroup's 16 keys per thread hold, so the 32-keys-per-thread instantiation ranks them.  One KV
    head; selection over every page and attention against the oracle, for a small and a large budget."""
    from paper_2604_10539_amd import IceIndex
    w = datagen.small("ctx300k", n_kv_heads=1, n_tokens=300000, n_clusters=2048, token_budget=1024, n_components=1024,
                      outlier_frac=0.05, seed=3300)
    K, V = datagen.keys_values(w)
    K, V = K.reshape(1, w.n_tokens, D), V.reshape(1, w.n_tokens, D)
    init, q_np = datagen.init_indices(w), datagen.queries(w)
    ix = IceIndex(1, 1, 4, w.n_tokens, 16, w.n_clusters, kmeans_iters=1, init_idx=up(init))
    ix.build_index(up(K), up(V))
    ex = ix.export()
    assert int(ex["n_pages"][0]) > 16384
    for budget in (1024, 256, 16 * 300):
        ids, n_sel, out = ix.select_attend(up(q_np), budget)
        torch.cuda.synchronize()
        _select_attend_vs_oracle(ix, ex, q_np, budget, ids, n_sel, out)
    _check_units(ix, ex, K, V, [0], w.n_tokens, np.random.default_rng(3), n_keys=32)


def test_thousands_of_tied_pages_are_ranked_from_the_registers():
    """More exactly tied candidates than the LDS candidate list holds (5000 identical pages, a few better
    and a few worse ones): the selection falls back to the radix select over the key registers and
    must still return the best pages, lowest ids first among the ties."""
    from paper_2604_10539_amd import IceIndex
    from tests.util import export_np, oracle_from_export
    rng = np.random.default_rng(19)
    n = 16 * 5000
    key = narrow(rng.standard_normal(D).astype(np.float32))
    K = np.tile(key, (1, 1, n, 1))
    K[0, 0, 16 * 4100:16 * 4103] = narrow(3.0 * widen(key))         # three pages that beat the rest
    K[0, 0, 16 * 10:16 * 12] = narrow(-1.0 * widen(key))            # two pages that lose
    V = narrow(rng.standard_normal((1, 1, n, D)).astype(np.float32))
    ix = IceIndex(1, 1, 1, n, 16, 1, kmeans_iters=1, init_idx=up(np.zeros((1, 1, 1), np.int32)))
    ix.build_index(up(K), up(V))
    q = narrow(widen(key)[None, None, :].copy())
    o = oracle_from_export(ix, export_np(ix))
    for pages in (8, 40, 200):
        ids, n_sel, scores = ix.select(up(q), 16 * pages)
        want = sorted([4100, 4101, 4102] + [p for p in range(pages) if p not in (10, 11)][:pages - 3])
        assert down(ids).ravel().tolist() == want, pages
        _compare_select(o, q, 16 * pages, down(ids), down(n_sel), down(scores))
