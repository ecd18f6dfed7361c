"""Pins for the CPU oracle: each test ties one oracle step to something that is not the oracle —
numpy brute force over the direct definition, a hand-written example, a closed form, an
invariant, or a library routine (torch SDPA).  CPU only."""
import math

import numpy as np
import pytest

import datagen
from datagen import bf16_bits_to_f32 as widen, f32_to_bf16_bits as narrow
from oracle import ice_oracle as orc

D = 128


def _rand_bits(rng, shape, scale=1.0):
    return narrow((scale * rng.standard_normal(shape)).astype(np.float32))


# ----------------------------------------------------------------------------- assign (Sec. 4.2)
@pytest.mark.parametrize("n,C,seed", [(64, 8, 0), (37, 5, 1), (500, 24, 2), (1, 1, 3)])
def test_assign_is_exhaustive_nearest_centroid(n, C, seed):
    """argmin over the full n x C matrix of ||k - mu||^2 computed directly (not the expanded form)."""
    rng = np.random.default_rng(seed)
    K = _rand_bits(rng, (n, D))
    mu = _rand_bits(rng, (C, D))
    a, best, second = orc.assign(K, mu)
    kf, mf = widen(K).astype(np.float64), widen(mu).astype(np.float64)
    dist = ((kf[:, None, :] - mf[None, :, :]) ** 2).sum(-1)
    assert np.array_equal(a, dist.argmin(1).astype(np.int32))
    # the objective drops the key's own norm: best + ||k||^2 is the true squared distance
    np.testing.assert_allclose(best + (kf ** 2).sum(1), dist.min(1), rtol=0, atol=1e-9)
    if C > 1:
        np.testing.assert_allclose(second + (kf ** 2).sum(1), np.sort(dist, 1)[:, 1], rtol=0, atol=1e-9)


def test_assign_ties_take_lowest_index():
    rng = np.random.default_rng(5)
    K = _rand_bits(rng, (40, D))
    mu = _rand_bits(rng, (3, D))
    mu6 = np.concatenate([mu, mu])            # centroid c+3 duplicates centroid c
    a, _, _ = orc.assign(K, mu6)
    assert a.max() <= 2
    a3, _, _ = orc.assign(K, mu)
    assert np.array_equal(a, a3)


def test_assign_key_equal_to_centroid_picks_it():
    rng = np.random.default_rng(6)
    mu = _rand_bits(rng, (16, D))
    a, best, _ = orc.assign(mu.copy(), mu)
    assert np.array_equal(a, np.arange(16))
    np.testing.assert_allclose(best + (widen(mu).astype(np.float64) ** 2).sum(1), 0.0, atol=1e-9)


# ----------------------------------------------------------------------------- means (Lloyd step)
def test_means_match_numpy_scatter_add_and_empty_cluster_keeps_centroid():
    rng = np.random.default_rng(7)
    n, C = 300, 9
    K = _rand_bits(rng, (n, D))
    a = rng.integers(0, C - 1, n).astype(np.int32)      # cluster C-1 stays empty
    prev = rng.standard_normal((C, D)).astype(np.float32)
    mu, ssum, cnt = orc.means(K, a, C, prev)
    acc = np.zeros((C, D))
    np.add.at(acc, a, widen(K).astype(np.float64))
    ref_cnt = np.bincount(a, minlength=C)
    assert np.array_equal(cnt, ref_cnt)
    np.testing.assert_allclose(ssum, acc, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(mu[:-1], acc[:-1] / ref_cnt[:-1, None], rtol=1e-6, atol=1e-6)
    assert np.array_equal(mu[-1], prev[-1])


# ----------------------------------------------------------------------------- Lloyd rounds
def _inertia(K, mu, a):
    kf = widen(K).astype(np.float64)
    return float(((kf - mu.astype(np.float64)[a]) ** 2).sum())


def test_lloyd_round1_is_nearest_promoted_key():
    """The first Lloyd round is the paper's two-level parent assignment: parent = nearest promoted key (Alg. 2)."""
    w = datagen.small(n_tokens=400, n_clusters=12)
    K, _ = datagen.keys_values(w)
    idx = datagen.init_indices(w)
    a, mu, ssum, cnt, _ = orc.lloyd(K[0, 0], idx[0, 0], 1)
    kf = widen(K[0, 0]).astype(np.float64)
    dist = ((kf[:, None, :] - kf[idx[0, 0]][None, :, :]) ** 2).sum(-1)
    assert np.array_equal(a, dist.argmin(1))
    assert np.array_equal(a[idx[0, 0]], np.arange(12))     # a promoted key is its own parent


def test_lloyd_final_state_invariants_and_monotone_inertia():
    w = datagen.small(n_tokens=800, n_clusters=20, n_components=10)
    K, _ = datagen.keys_values(w)
    idx = datagen.init_indices(w)
    T = 6
    a, mu, ssum, cnt, inertia = orc.lloyd(K[0, 1], idx[0, 1], T)
    kf = widen(K[0, 1]).astype(np.float64)
    # centroids are the means of the final assignment
    for c in range(20):
        m = a == c
        assert cnt[c] == m.sum()
        if m.any():
            np.testing.assert_allclose(mu[c], kf[m].mean(0), rtol=1e-6, atol=1e-6)
            np.testing.assert_allclose(ssum[c], kf[m].sum(0), rtol=1e-6, atol=1e-5)
    assert cnt.sum() == 800
    # k-means never increases the objective (up to the bf16 rounding of the centroids)
    assert np.all(np.diff(inertia) <= 1e-3 * inertia[:-1])
    assert inertia[-1] < inertia[0]
    # the reported inertia is the objective seen by that round's assignment
    a1, mu1, *_ = orc.lloyd(K[0, 1], idx[0, 1], 1)
    mu0 = widen(narrow(widen(K[0, 1][idx[0, 1]])))
    np.testing.assert_allclose(inertia[0], _inertia(K[0, 1], mu0, a1), rtol=1e-9)


def test_lloyd_recovers_well_separated_components():
    """Special case with a known answer: one promoted key per far-apart component."""
    rng = np.random.default_rng(11)
    M, per = 6, 30
    cen = 20.0 * np.eye(M, D, dtype=np.float32)
    lab = np.repeat(np.arange(M), per)
    x = cen[lab] + 0.1 * rng.standard_normal((M * per, D)).astype(np.float32)
    K = narrow(x)
    init = np.arange(M, dtype=np.int32) * per
    a, mu, _, cnt, _ = orc.lloyd(K, init, 3)
    assert np.array_equal(a, lab)
    assert np.all(cnt == per)
    np.testing.assert_allclose(mu, cen, atol=0.1)


def test_lloyd_equals_composed_steps():
    w = datagen.small(n_tokens=300, n_clusters=7)
    K, _ = datagen.keys_values(w)
    idx = datagen.init_indices(w)
    a, mu, ssum, cnt, _ = orc.lloyd(K[0, 0], idx[0, 0], 3)
    m = widen(K[0, 0][idx[0, 0]]).copy()
    for _ in range(3):
        aa, _, _ = orc.assign(K[0, 0], narrow(m))
        m, ss, cc = orc.means(K[0, 0], aa, 7, m)
    assert np.array_equal(a, aa) and np.array_equal(mu, m) and np.array_equal(cnt, cc)


# ----------------------------------------------------------------------------- pages (Sec. 4.1)
def test_paginate_hand_example():
    """n = 10, s = 4, C = 3, written out by hand."""
    rng = np.random.default_rng(13)
    K = _rand_bits(rng, (1, 10, D))
    V = _rand_bits(rng, (1, 10, D))
    a = np.array([[2, 0, 2, 2, 0, 2, 2, 0, 2, 2]], np.int32)   # cluster 1 is empty
    ix = orc.OracleIndex(1, 1, 4, 3, max_tokens=16)
    ix.paginate(K, V, a)
    # cluster 0: tokens 1,4,7 -> page 0; cluster 2: tokens 0,2,3,5 -> page 1; 6,8,9 -> page 2
    assert ix.n_pages[0] == 3 and ix.n_tokens[0] == 10
    assert ix.page_cluster[0, :4].tolist() == [0, 2, 2, -1]
    assert ix.page_fill[0, :4].tolist() == [3, 4, 3, 0]
    assert ix.page_pos[0, :3].tolist() == [[1, 4, 7, -1], [0, 2, 3, 5], [6, 8, 9, -1]]
    assert ix.cluster_tail[0].tolist() == [0, -1, 2]
    assert np.array_equal(ix.Kp[0, 1, 2], K[0, 3]) and np.array_equal(ix.Vp[0, 2, 0], V[0, 6])
    # representative of page 0 = mean of keys 1,4,7 up to bf16 rounding
    mean = widen(K[0, [1, 4, 7]]).astype(np.float64).mean(0)
    got = widen(ix.rep[0, 0]).astype(np.float64)
    assert np.all(np.abs(got - mean) <= np.abs(mean) * 2.0 ** -8 + 1e-30)
    s3 = widen(K[0, 1]) + widen(K[0, 4])
    s3 = s3 + widen(K[0, 7])
    assert np.array_equal(ix.page_sum[0, 0], s3)               # slot order, fp32


def _check_invariants(ix, K_all, V_all, assign_all):
    """I1-I4, I6 on an OracleIndex; K_all/V_all [U, n, d], assign_all [U, n]."""
    for u in range(ix.U):
        n, npg = int(ix.n_tokens[u]), int(ix.n_pages[u])
        fill = ix.page_fill[u, :npg]
        assert fill.sum() == n and fill.min() >= 1 and fill.max() <= ix.s            # I2
        pos = ix.page_pos[u, :npg]
        valid = np.arange(ix.s)[None, :] < fill[:, None]
        assert np.array_equal(np.sort(pos[valid]), np.arange(n))                      # I1
        assert np.all(pos[~valid] == -1)
        for c in range(ix.C):
            pages = np.nonzero(ix.page_cluster[u, :npg] == c)[0]
            partial = pages[fill[pages] < ix.s]
            assert len(partial) <= 1                                                  # I3
            if len(pages):
                assert ix.cluster_tail[u, c] == pages.max()
                if len(partial):
                    assert partial[0] == pages.max()
            else:
                assert ix.cluster_tail[u, c] == -1
        pc = np.repeat(ix.page_cluster[u, :npg], ix.s).reshape(npg, ix.s)
        assert np.array_equal(assign_all[u][pos[valid]], pc[valid])                   # I4
        assert np.array_equal(ix.Kp[u, :npg][valid], K_all[u][pos[valid]])            # I6
        assert np.array_equal(ix.Vp[u, :npg][valid], V_all[u][pos[valid]])


def test_paginate_invariants_random():
    w = datagen.small(n_tokens=777, n_clusters=19, n_kv_heads=3)
    K, V = datagen.keys_values(w)
    rng = np.random.default_rng(17)
    a = rng.integers(0, 19, (3, 777)).astype(np.int32)
    ix = orc.OracleIndex(3, 4, 16, 19, max_tokens=800)
    ix.paginate(K[0], V[0], a)
    _check_invariants(ix, K[0], V[0], a)
    # within a cluster tokens appear in ascending position and pages are consecutive
    for u in range(3):
        npg = ix.n_pages[u]
        assert np.all(np.diff(ix.page_cluster[u, :npg]) >= 0)
        for c in range(19):
            pages = np.nonzero(ix.page_cluster[u, :npg] == c)[0]
            seq = [p for pg in pages for p in ix.page_pos[u, pg] if p >= 0]
            assert seq == sorted(seq) and seq == np.nonzero(a[u] == c)[0].tolist()


def test_representative_of_identical_keys_is_the_key():
    """fill copies of one bf16 vector: the fp32 sum and the divide are exact, so rep == key bits."""
    rng = np.random.default_rng(19)
    key = _rand_bits(rng, (D,))
    for fill in (1, 2, 5, 16):
        K = np.tile(key, (1, fill, 1))
        ix = orc.OracleIndex(1, 1, 16, 1, max_tokens=16)
        ix.paginate(K, K, np.zeros((1, fill), np.int32))
        assert np.array_equal(ix.rep[0, 0], key)
        np.testing.assert_array_equal(ix.page_sum[0, 0], fill * widen(key))


def test_representative_is_rounded_mean():
    rng = np.random.default_rng(23)
    K = _rand_bits(rng, (1, 16 * 5, D))
    ix = orc.OracleIndex(1, 1, 16, 1, max_tokens=80)
    ix.paginate(K, K, np.zeros((1, 80), np.int32))
    mean = widen(K[0]).astype(np.float64).reshape(5, 16, D).mean(1)
    got = widen(ix.rep[0, :5]).astype(np.float64)
    # fp32 sum of 16 terms then one bf16 rounding: half a bf16 ulp (<= 2^-8 relative) plus the sum error
    assert np.all(np.abs(got - mean) <= np.abs(mean) * 2.0 ** -8 + 1e-5)


# ----------------------------------------------------------------------------- insert (Alg. 1, Sec. 4.2)
def test_insert_follows_nearest_centroid_and_keeps_invariants():
    w = datagen.small(n_tokens=640, n_clusters=10, n_kv_heads=2, n_components=8)
    K, V = datagen.keys_values(w, n_tokens=700)
    idx = datagen.init_indices(w, n_tokens=600)
    ix = orc.OracleIndex(2, 4, 16, 10, max_tokens=700)
    ix.build(K[0, :, :600], V[0, :, :600], idx[0], 4)
    assign = [ix.assign[u].tolist() for u in range(2)]
    for t in range(600, 700):
        mub = narrow(ix.centroid)                         # centroids as seen by this insertion
        pages_before = ix.n_pages.copy()
        tails = ix.cluster_tail.copy()
        fills = ix.page_fill.copy()
        chosen, best, second = ix.insert(K[0, :, t], V[0, :, t])
        for u in range(2):
            kf = widen(K[0, u, t]).astype(np.float64)
            dist = ((kf[None, :] - widen(mub[u]).astype(np.float64)) ** 2).sum(-1)
            assert chosen[u] == dist.argmin()
            c = int(chosen[u])
            assign[u].append(c)
            old_tail = tails[u, c]
            if old_tail < 0 or fills[u, old_tail] == 16:   # node outgrew its page: a new page
                assert ix.n_pages[u] == pages_before[u] + 1
                assert ix.cluster_tail[u, c] == pages_before[u]
                assert ix.page_fill[u, pages_before[u]] == 1
            else:
                assert ix.n_pages[u] == pages_before[u]
                assert ix.page_fill[u, old_tail] == fills[u, old_tail] + 1
    a = np.array(assign, np.int32)
    _check_invariants(ix, K[0], V[0], a)
    kf = widen(K[0]).astype(np.float64)
    for u in range(2):
        for c in range(10):
            m = a[u] == c
            assert ix.cluster_cnt[u, c] == m.sum()
            if m.any():                                    # running mean == true mean (I5)
                np.testing.assert_allclose(ix.centroid[u, c], kf[u][m].mean(0), rtol=1e-5, atol=1e-5)
    # representatives stay the rounded mean of their page
    for u in range(2):
        for p in range(ix.n_pages[u]):
            f = ix.page_fill[u, p]
            mean = widen(ix.Kp[u, p, :f]).astype(np.float64).mean(0)
            got = widen(ix.rep[u, p]).astype(np.float64)
            assert np.all(np.abs(got - mean) <= np.abs(mean) * 2.0 ** -8 + 1e-5)


def test_insert_into_empty_cluster_and_capacity():
    rng = np.random.default_rng(29)
    K = _rand_bits(rng, (1, 8, D))
    ix = orc.OracleIndex(1, 1, 4, 2, max_tokens=9)
    ix.paginate(K, K, np.zeros((1, 8), np.int32))          # cluster 1 owns nothing
    ix.centroid[0, 0] = widen(K[0]).mean(0)
    ix.cluster_cnt[0] = [8, 0]
    far = narrow(np.full(D, 50.0, np.float32))
    ix.centroid[0, 1] = widen(far)
    chosen, _, _ = ix.insert(far[None], far[None])
    assert chosen[0] == 1 and ix.n_pages[0] == 3 and ix.cluster_tail[0, 1] == 2
    assert ix.page_pos[0, 2, 0] == 8 and ix.page_fill[0, 2] == 1
    assert np.array_equal(ix.rep[0, 2], far) and ix.cluster_cnt[0, 1] == 1
    with pytest.raises(OverflowError):
        ix.insert(far[None], far[None])


def test_insert_force_overrides_choice():
    rng = np.random.default_rng(31)
    K = _rand_bits(rng, (1, 8, D))
    ix = orc.OracleIndex(1, 1, 4, 2, max_tokens=16)
    ix.paginate(K, K, (np.arange(8) % 2)[None].astype(np.int32))
    ix.centroid[0] = 0
    chosen, _, _ = ix.insert(K[0, :1], K[0, :1], force=np.array([1], np.int32))
    assert chosen[0] == 1 and ix.page_cluster[0, ix.n_pages[0] - 1] == 1


# ----------------------------------------------------------------------------- select (Sec. 4.4, Alg. 3)
def _built(w, T=3, max_extra=0):
    K, V = datagen.keys_values(w)
    idx = datagen.init_indices(w)
    U = w.batch * w.n_kv_heads
    ix = orc.OracleIndex(U, w.group_size, w.page_size, w.n_clusters, max_tokens=w.n_tokens + max_extra)
    ix.build(K, V, idx, T)
    return ix, K.reshape(U, w.n_tokens, D), V.reshape(U, w.n_tokens, D)


def _scores_numpy(ix, q):
    qf = widen(q).astype(np.float64)                       # [U, G, d]
    out = []
    for u in range(ix.U):
        r = widen(ix.rep[u, :ix.n_pages[u]]).astype(np.float64)
        sc = (r @ qf[u].T) / np.linalg.norm(qf[u], axis=1)[None, :]
        out.append(sc.max(1).astype(np.float32))
    return out


@pytest.mark.parametrize("budget", [16, 128, 256])
def test_select_is_full_sort(budget):
    w = datagen.small(n_tokens=1500, n_clusters=24, n_kv_heads=3)
    ix, _, _ = _built(w)
    q = datagen.queries(w).reshape(ix.U, w.group_size, D)
    ids, n_sel, scores, S_all = ix.select(q, budget)
    P = budget // 16
    S = _scores_numpy(ix, q)
    for u in range(ix.U):
        npg = int(ix.n_pages[u])
        np.testing.assert_allclose(S_all[u, :npg], S[u], rtol=2e-7, atol=1e-7)
        order = sorted(range(npg), key=lambda p: (-S_all[u, p], p))
        want = sorted(order[:min(P, npg)])
        assert n_sel[u] == len(want)
        assert ids[u, :len(want)].tolist() == want
        assert np.all(ids[u, len(want):] == -1)
        assert np.array_equal(scores[u, :len(want)], S_all[u, want])
        assert ix.page_fill[u, want].sum() <= budget       # loaded keys <= pages x page size


def test_select_budget_covering_everything_returns_every_page():
    w = datagen.small(n_tokens=300, n_clusters=6)
    ix, _, _ = _built(w)
    q = datagen.queries(w).reshape(ix.U, w.group_size, D)
    ids, n_sel, _, _ = ix.select(q, 16 * 64)
    for u in range(ix.U):
        assert n_sel[u] == ix.n_pages[u]
        assert ids[u, :n_sel[u]].tolist() == list(range(ix.n_pages[u]))


def test_select_ties_take_lowest_page_id():
    rng = np.random.default_rng(37)
    key = _rand_bits(rng, (D,))
    K = np.tile(key, (1, 64, 1))                           # 4 identical pages
    ix = orc.OracleIndex(1, 2, 16, 1, max_tokens=64)
    ix.paginate(K, K, np.zeros((1, 64), np.int32))
    q = _rand_bits(rng, (1, 2, D))
    ids, n_sel, _, _ = ix.select(q, 32)
    assert n_sel[0] == 2 and ids[0].tolist() == [0, 1]


def test_select_single_token_pages_rank_like_the_transformed_euclidean_search():
    """With one key per page the representative is the key, and ranking by q.k/||q|| must equal
    ranking by Euclidean distance between T_K(k) and T_Q(q) (Eqs. 2-3):
    ||T_K(k) - T_Q(q)||^2 = 2 - 2 q.k / (c ||q||)."""
    rng = np.random.default_rng(41)
    n = 48
    K = _rand_bits(rng, (1, n, D))
    ix = orc.OracleIndex(1, 1, 16, n, max_tokens=n)
    ix.paginate(K, K, np.arange(n, dtype=np.int32)[None])  # every token its own node
    q = _rand_bits(rng, (1, 1, D))
    ids, n_sel, _, _ = ix.select(q, 16 * 5)
    kf, qf = widen(K[0]).astype(np.float64), widen(q[0, 0]).astype(np.float64)
    c = np.linalg.norm(kf, axis=1).max() * 1.01
    TK = np.concatenate([kf / c, np.sqrt(1 - (kf ** 2).sum(1) / c ** 2)[:, None]], 1)
    TQ = np.concatenate([qf / np.linalg.norm(qf), [0.0]])
    dist = ((TK - TQ[None]) ** 2).sum(1)
    np.testing.assert_allclose(dist, 2 - 2 * (kf @ qf) / (c * np.linalg.norm(qf)), atol=1e-12)
    assert ids[0].tolist() == sorted(np.argsort(dist)[:5].tolist())


def test_select_group_score_is_max_over_heads():
    """A page that only one query head of the group likes is still selected (GQA sharing, Sec. 4.3)."""
    e = np.zeros((3, D), np.float32)
    e[0, 0] = e[1, 1] = e[2, 2] = 4.0
    K = narrow(np.repeat(e, 16, axis=0))[None]             # three pages along three axes
    ix = orc.OracleIndex(1, 2, 16, 3, max_tokens=48)
    ix.paginate(K, K, np.repeat(np.arange(3), 16)[None].astype(np.int32))
    qv = np.zeros((1, 2, D), np.float32)
    qv[0, 0, 0] = 1.0
    qv[0, 0, 2] = 0.5
    qv[0, 1, 1] = 100.0                                    # a long query must not dominate: scores are normalised
    qv[0, 1, 2] = 60.0
    ids, n_sel, scores, S_all = ix.select(narrow(qv), 32)
    # head 0 scores (4/|q0|, 0, 2/|q0|) = (3.578, 0, 1.789); head 1 scores (0, 3.43, 2.058)
    assert ids[0].tolist() == [0, 1]
    np.testing.assert_allclose(S_all[0, :3], [4 / math.hypot(1, .5), 400 / math.hypot(100, 60),
                                              240 / math.hypot(100, 60)], rtol=1e-6)


# ----------------------------------------------------------------------------- attend (Eq. 1)
def _dense_attention(q, K, V):
    """Textbook softmax attention, fp64: q [G,d], K,V [n,d]."""
    z = (q @ K.T) / math.sqrt(q.shape[-1])
    z = z - z.max(1, keepdims=True)
    p = np.exp(z)
    return (p / p.sum(1, keepdims=True)) @ V


def test_attend_with_every_page_equals_dense_attention():
    w = datagen.small(n_tokens=900, n_clusters=12, n_kv_heads=2)
    ix, K, V = _built(w)
    q = datagen.queries(w).reshape(ix.U, w.group_size, D)
    ids, n_sel, _, _ = ix.select(q, 16 * 128)
    out = ix.attend(q, ids, n_sel)
    import torch
    for u in range(ix.U):
        ref = _dense_attention(widen(q[u]).astype(np.float64), widen(K[u]).astype(np.float64),
                               widen(V[u]).astype(np.float64))
        np.testing.assert_allclose(out[u], ref, rtol=0, atol=2e-7 * max(1.0, np.abs(ref).max()))
        tq = torch.from_numpy(widen(q[u]).copy())[None]
        sd = torch.nn.functional.scaled_dot_product_attention(
            tq, torch.from_numpy(widen(K[u]).copy())[None], torch.from_numpy(widen(V[u]).copy())[None])
        np.testing.assert_allclose(out[u], sd[0].numpy(), rtol=0, atol=2e-5)


def test_attend_subset_equals_dense_attention_over_that_subset():
    w = datagen.small(n_tokens=900, n_clusters=12, n_kv_heads=2)
    ix, K, V = _built(w)
    q = datagen.queries(w).reshape(ix.U, w.group_size, D)
    ids, n_sel, _, _ = ix.select(q, 64)
    out = ix.attend(q, ids, n_sel)
    for u in range(ix.U):
        pos = np.concatenate([ix.page_pos[u, p, :ix.page_fill[u, p]] for p in ids[u, :n_sel[u]]])
        ref = _dense_attention(widen(q[u]).astype(np.float64), widen(K[u][pos]).astype(np.float64),
                               widen(V[u][pos]).astype(np.float64))
        np.testing.assert_allclose(out[u], ref, rtol=0, atol=2e-7 * max(1.0, np.abs(ref).max()))
        # the order in which the pages are listed does not matter
        perm = ids[u, :n_sel[u]][::-1].copy()
        ids2 = ids.copy()
        ids2[u, :n_sel[u]] = perm
        np.testing.assert_allclose(ix.attend(q, ids2, n_sel)[u], out[u], rtol=0, atol=1e-6)


def test_attend_closed_forms():
    rng = np.random.default_rng(43)
    key = _rand_bits(rng, (D,))
    V = _rand_bits(rng, (1, 40, D))
    K = np.tile(key, (1, 40, 1))
    ix = orc.OracleIndex(1, 3, 16, 1, max_tokens=40)
    ix.paginate(K, V, np.zeros((1, 40), np.int32))
    q = _rand_bits(rng, (1, 3, D))
    # all keys equal -> uniform weights -> mean of the values
    out = ix.attend(q, np.array([[0, 1, 2]], np.int32), np.array([3], np.int32))
    np.testing.assert_allclose(out[0], np.tile(widen(V[0]).astype(np.float64).mean(0), (3, 1)), atol=1e-6)
    # one page holding the ragged tail (8 tokens)
    out = ix.attend(q, np.array([[2, -1, -1]], np.int32), np.array([1], np.int32))
    np.testing.assert_allclose(out[0], np.tile(widen(V[0, 32:]).astype(np.float64).mean(0), (3, 1)), atol=1e-6)
    # nothing selected -> zeros
    out = ix.attend(q, np.array([[-1, -1, -1]], np.int32), np.array([0], np.int32))
    assert np.all(out == 0)
    # one page with one token -> that token's value
    ix1 = orc.OracleIndex(1, 3, 16, 1, max_tokens=16)
    ix1.paginate(K[:, :1], V[:, :1], np.zeros((1, 1), np.int32))
    out = ix1.attend(q, np.array([[0]], np.int32), np.array([1], np.int32))
    np.testing.assert_array_equal(out[0], np.tile(widen(V[0, 0]), (3, 1)))


def test_attend_two_tokens_is_a_sigmoid_of_the_scaled_logit_gap():
    """Pins the 1/sqrt(d) scale: weights of two keys are sigmoid(+-(q.k1 - q.k2)/sqrt(d))."""
    k = np.zeros((2, D), np.float32)
    k[0, 0], k[1, 0] = 3.0, -1.0
    v = np.zeros((2, D), np.float32)
    v[0, 5], v[1, 5] = 1.0, 0.0
    ix = orc.OracleIndex(1, 1, 16, 1, max_tokens=16)
    ix.paginate(narrow(k)[None], narrow(v)[None], np.zeros((1, 2), np.int32))
    q = np.zeros((1, 1, D), np.float32)
    q[0, 0, 0] = 2.0
    out = ix.attend(narrow(q), np.array([[0]], np.int32), np.array([1], np.int32))
    gap = (2.0 * 3.0 - 2.0 * (-1.0)) / math.sqrt(D)
    assert abs(out[0, 0, 5] - 1.0 / (1.0 + math.exp(-gap))) < 1e-7


# ----------------------------------------------------------------------------- input recipe sanity
def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2.0 ** -9, -2.5, 3.0e38], np.float32)
    got = widen(narrow(x))
    # 1 + 2^-8 lies halfway between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 -> 1 + 2^-6 (even)
    assert got.tolist()[:5] == [1.0, 1.0, 1.015625, 1.0, -2.5]
    import torch
    y = np.random.default_rng(1).standard_normal(10000).astype(np.float32)
    ref = torch.from_numpy(y).to(torch.bfloat16).float().numpy()
    assert np.array_equal(widen(narrow(y)), ref)


# ----------------------------------------------------------------------------- hierarchical select (Sec. 3.3, Alg. 4)
def _hier_numpy(ix, q, budget, n_probe):
    """The staged definition written out with numpy and Python sorting (fp64 scores rounded to fp32)."""
    qf = widen(q).astype(np.float64)
    P = budget // ix.s
    out = []
    for u in range(ix.U):
        mu = widen(narrow(ix.centroid[u])).astype(np.float64)                  # bf16-rounded centroids
        nq = np.linalg.norm(qf[u], axis=1)[None, :]
        sc = ((mu @ qf[u].T) / nq).max(1).astype(np.float32)
        kept = sorted(sorted(range(ix.C), key=lambda c: (-sc[c], c))[:min(n_probe, ix.C)])
        npg = int(ix.n_pages[u])
        cand = [p for p in range(npg) if ix.page_cluster[u, p] in set(kept)]
        r = widen(ix.rep[u, :npg]).astype(np.float64)
        sp = ((r @ qf[u].T) / nq).max(1).astype(np.float32)
        best = sorted(sorted(cand, key=lambda p: (-sp[p], p))[:min(P, len(cand))])
        out.append((kept, best, sc))
    return out


@pytest.mark.parametrize("n_probe,budget", [(1, 64), (4, 64), (8, 256), (24, 128)])
def test_hier_select_is_the_staged_definition(n_probe, budget):
    w = datagen.small(n_tokens=1500, n_clusters=24, n_kv_heads=3)
    ix, _, _ = _built(w)
    q = datagen.queries(w).reshape(ix.U, w.group_size, D)
    ids, n_sel, scores, clusters, Sc_all = ix.select_hier(q, budget, n_probe)
    _, _, _, S_all = ix.select(q, budget)
    for u, (kept, best, sc) in enumerate(_hier_numpy(ix, q, budget, n_probe)):
        np.testing.assert_allclose(Sc_all[u], sc, rtol=2e-7, atol=1e-7)
        assert clusters[u, :len(kept)].tolist() == kept and np.all(clusters[u, len(kept):] == -1)
        assert n_sel[u] == len(best) and ids[u, :len(best)].tolist() == best
        assert np.all(ids[u, len(best):] == -1)
        assert np.array_equal(scores[u, :len(best)], S_all[u, best])
        # every returned page belongs to a kept cluster
        assert set(ix.page_cluster[u, best].tolist()) <= set(kept)


def test_hier_select_with_every_cluster_is_the_flat_select():
    w = datagen.small(n_tokens=2000, n_clusters=20, n_kv_heads=2)
    ix, _, _ = _built(w)
    q = datagen.queries(w).reshape(ix.U, w.group_size, D)
    for n_probe in (20, 64):                                # == C and > C
        ids_h, ns_h, sc_h, clusters, _ = ix.select_hier(q, 128, n_probe)
        ids_f, ns_f, sc_f, _ = ix.select(q, 128)
        assert np.array_equal(ids_h, ids_f) and np.array_equal(ns_h, ns_f) and np.array_equal(sc_h, sc_f)
        assert np.array_equal(clusters[:, :20], np.tile(np.arange(20), (ix.U, 1)))


def test_hier_select_one_cluster_returns_only_its_pages():
    """n_probe = 1: the answer is the best pages of the single cluster whose centroid the query likes most;
    with a budget that covers that cluster, exactly its pages come back."""
    w = datagen.small(n_tokens=1200, n_clusters=10, n_kv_heads=2)
    ix, _, _ = _built(w)
    q = datagen.queries(w).reshape(ix.U, w.group_size, D)
    ids, n_sel, _, clusters, Sc_all = ix.select_hier(q, 16 * 200, 1)
    for u in range(ix.U):
        c = int(clusters[u, 0])
        assert c == int(np.lexsort((np.arange(ix.C), -Sc_all[u]))[0])
        mine = [p for p in range(ix.n_pages[u]) if ix.page_cluster[u, p] == c]
        assert ids[u, :n_sel[u]].tolist() == mine


def test_hier_select_sees_pages_appended_by_insertion():
    """Pages opened by later insertions sit at the end of the page range, not next to their cluster's
    build-time pages; they must still be candidates of their cluster."""
    w = datagen.small(n_tokens=640, n_clusters=4, n_kv_heads=1, n_components=4)
    ix, _, _ = _built(w, max_extra=256)
    np0 = int(ix.n_pages[0])
    stream = datagen.DecodeStream(w, seed=3)
    for _ in range(200):
        k, v, _ = stream.next()
        ix.insert(k, v)
    assert ix.n_pages[0] > np0
    c = int(ix.page_cluster[0, ix.n_pages[0] - 1])          # a cluster that owns an appended page
    q = np.tile(narrow(ix.centroid[0, c])[None, None, :], (1, w.group_size, 1))   # a query along its centroid
    ids, n_sel, _, clusters, _ = ix.select_hier(q, 16 * 400, 1)
    assert int(clusters[0, 0]) == c
    mine = [p for p in range(ix.n_pages[0]) if ix.page_cluster[0, p] == c]
    assert any(p >= np0 for p in mine)                      # the case under test exists
    assert ids[0, :n_sel[0]].tolist() == mine


def test_refined_selection_ranks_pages_by_their_best_key():
    """Stage 3 written out with numpy: of the n_refine best pages by representative, those holding the
    best keys win; with n_refine = 0 nothing changes, and with one token per page (representative ==
    key) refinement cannot change the order."""
    w = datagen.small(n_tokens=1800, n_clusters=20, n_kv_heads=2)
    ix, _, _ = _built(w)
    q = datagen.queries(w).reshape(ix.U, w.group_size, D)
    budget, n_refine = 64, 24
    P = budget // 16
    ids, n_sel, scores, _, _ = ix.select_hier(q, budget, ix.C, n_refine)
    _, _, _, S_all = ix.select(q, budget)
    qf = widen(q).astype(np.float64)
    changed = 0
    for u in range(ix.U):
        npg = int(ix.n_pages[u])
        kept = sorted(range(npg), key=lambda p: (-S_all[u, p], p))[:n_refine]
        nq = np.linalg.norm(qf[u], axis=1)
        best = {}
        for p in kept:
            kk = widen(ix.Kp[u, p, :ix.page_fill[u, p]]).astype(np.float64)
            best[p] = np.float32(((kk @ qf[u].T) / nq[None, :]).max())
        want = sorted(sorted(kept, key=lambda p: (-best[p], p))[:P])
        assert ids[u, :n_sel[u]].tolist() == want
        np.testing.assert_allclose(scores[u, :n_sel[u]], [best[p] for p in want], rtol=3e-7)
        changed += want != sorted(kept[:P])
        assert all(best[p] >= S_all[u, p] - 0.01 * abs(S_all[u, p]) - 1e-5 for p in kept)   # best key >= mean key (bf16 rep)
    assert changed > 0                                              # the case is not vacuous
    a = ix.select_hier(q, budget, ix.C, 0)
    f = ix.select(q, budget)
    assert np.array_equal(a[0], f[0]) and np.array_equal(a[2], f[2])


# ----------------------------------------------------------------------------- attention with resident tokens
def test_attend_resident_is_dense_attention_over_the_union():
    """Selected pages + resident (sink / window) tokens: one softmax over their union, checked
    against torch's scaled_dot_product_attention on the gathered rows; with no resident tokens it is
    attend(); with no pages it is dense attention over the resident tokens alone."""
    import torch
    w = datagen.small(n_tokens=800, n_clusters=10, n_kv_heads=2)
    ix, K, V = _built(w)
    rng = np.random.default_rng(77)
    q = datagen.queries(w).reshape(ix.U, w.group_size, D)
    ids, n_sel, _, _ = ix.select(q, 64)
    n_res = 37
    rk, rv = _rand_bits(rng, (ix.U, n_res, D)), _rand_bits(rng, (ix.U, n_res, D))
    out = ix.attend_resident(q, ids, n_sel, rk, rv)
    for u in range(ix.U):
        rows_k, rows_v = [], []
        for p in ids[u, :n_sel[u]]:
            f = ix.page_fill[u, p]
            rows_k.append(ix.Kp[u, p, :f])
            rows_v.append(ix.Vp[u, p, :f])
        kk = torch.from_numpy(widen(np.concatenate(rows_k + [rk[u]])).astype(np.float64))
        vv = torch.from_numpy(widen(np.concatenate(rows_v + [rv[u]])).astype(np.float64))
        qq = torch.from_numpy(widen(q[u]).astype(np.float64))
        ref = torch.nn.functional.scaled_dot_product_attention(qq[None], kk[None], vv[None])[0].numpy()
        np.testing.assert_allclose(out[u], ref, rtol=0, atol=2e-6)
    none_k = np.zeros((ix.U, 0, D), np.uint16)
    assert np.array_equal(ix.attend_resident(q, ids, n_sel, none_k, none_k), ix.attend(q, ids, n_sel))
    only = ix.attend_resident(q, ids, np.zeros_like(n_sel), rk, rv)
    for u in range(ix.U):
        z = widen(q[u]).astype(np.float64) @ widen(rk[u]).astype(np.float64).T / math.sqrt(D)
        p = np.exp(z - z.max(1, keepdims=True))
        np.testing.assert_allclose(only[u], (p / p.sum(1, keepdims=True)) @ widen(rv[u]).astype(np.float64), atol=2e-6)


# ----------------------------------------------------------------------------- selection reuse by position
def test_attending_by_token_position_equals_attending_by_page():
    """The positions of the selected pages' tokens, applied to the cache the index was built from, give
    the page attention (the tiles are bit copies of those rows); applied to ANOTHER cache they give
    dense attention over those rows of that cache (checked with torch SDPA)."""
    import torch
    w = datagen.small(n_tokens=1100, n_clusters=14, n_kv_heads=2)
    ix, K, V = _built(w)
    q = datagen.queries(w).reshape(ix.U, w.group_size, D)
    ids, n_sel, _, _ = ix.select(q, 96)
    pos, n_tok = ix.selected_tokens(ids, n_sel)
    for u in range(ix.U):
        want = [int(t) for p in ids[u, :n_sel[u]] for t in ix.page_pos[u, p, :ix.page_fill[u, p]]]
        assert pos[u, :n_tok[u]].tolist() == want and np.all(pos[u, n_tok[u]:] == -1)
        assert len(set(want)) == len(want) and min(want) >= 0 and max(want) < w.n_tokens
    same = orc.attend_tokens(q, K, V, pos, n_tok)
    np.testing.assert_allclose(same, ix.attend(q, ids, n_sel), rtol=0, atol=1e-7)
    rng = np.random.default_rng(3)
    K2, V2 = _rand_bits(rng, K.shape), _rand_bits(rng, V.shape)          # "the next layer's" cache
    other = orc.attend_tokens(q, K2, V2, pos, n_tok)
    for u in range(ix.U):
        rows = pos[u, :n_tok[u]]
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(widen(q[u]).astype(np.float64))[None],
            torch.from_numpy(widen(K2[u, rows]).astype(np.float64))[None],
            torch.from_numpy(widen(V2[u, rows]).astype(np.float64))[None])[0].numpy()
        np.testing.assert_allclose(other[u], ref, rtol=0, atol=2e-6)


# ----------------------------------------------------------------------------- transformed keys (Eq. 2)
def test_transformed_key_distance_identity_and_unit_sphere():
    """c T_K(k) = [k, a] lies on the sphere of radius c, and squared distances between transformed keys are
    2 c^2 - 2 k_i.k_j - 2 a_i a_j (up to the bf16 rounding of a, which the identity is checked without)."""
    rng = np.random.default_rng(91)
    K = _rand_bits(rng, (2, 300, D), scale=2.0)
    extra, c2 = orc.key_extra_coordinate(K)
    kf = widen(K).astype(np.float64)
    n2 = (kf ** 2).sum(-1)
    np.testing.assert_allclose(c2, n2.max(-1))
    a = np.sqrt(np.maximum(c2[:, None] - n2, 0))
    np.testing.assert_allclose(widen(extra), a, rtol=2 ** -8, atol=1e-30)          # bf16 RNE of a
    T = np.concatenate([kf, a[..., None]], -1)
    np.testing.assert_allclose((T ** 2).sum(-1), np.broadcast_to(c2[:, None], n2.shape), rtol=1e-12)
    i, j = rng.integers(0, 300, 50), rng.integers(0, 300, 50)
    d2 = ((T[0, i] - T[0, j]) ** 2).sum(-1)
    np.testing.assert_allclose(d2, 2 * c2[0] - 2 * (kf[0, i] * kf[0, j]).sum(-1) - 2 * a[0, i] * a[0, j], atol=1e-9)
    # a key beyond the radius (inserted later) gets 0
    far = narrow((4.0 * widen(K[:, :1])).astype(np.float32))
    assert np.all(orc.key_extra_coordinate(far, c2)[0] == 0)


def test_transformed_keys_with_equal_norms_cluster_like_raw_keys():
    """When every key has the same norm the extra coordinate is the same for all keys and centroids'
    extra coordinates cancel out of every comparison: Lloyd on the transformed keys = Lloyd on the raw keys.
    (Keys are axis-aligned +-r vectors so that the norms are exactly equal in bf16.)"""
    rng = np.random.default_rng(92)
    n, C = 400, 6
    K = np.zeros((n, D), np.float32)
    K[np.arange(n), rng.integers(0, D, n)] = 3.0
    K[np.arange(n), rng.integers(0, D, n)] += 4.0 * (rng.integers(0, 2, n) * 2 - 1)   # |k|^2 in {25, 49, 1}: not equal yet
    K = K / np.linalg.norm(K, axis=1, keepdims=True)                                 # unit norm in fp32 ...
    Kb = narrow(K * 8.0)[None]                                                       # ... only nearly in bf16
    extra, c2 = orc.key_extra_coordinate(Kb)
    extra[:] = extra.max()                                                           # make the case exact: same a for all
    init = rng.choice(n, C, replace=False).astype(np.int32)
    a_raw, mu_raw, _, cnt_raw, _ = orc.lloyd(Kb[0], init, 4)
    a_tk, mu_tk, _, cnt_tk, _ = orc.lloyd(orc.augment(Kb, extra)[0], init, 4)
    assert np.array_equal(a_raw, a_tk) and np.array_equal(cnt_raw, cnt_tk)
    np.testing.assert_allclose(mu_tk[:, :D], mu_raw, rtol=0, atol=0)
    live = cnt_tk > 0
    np.testing.assert_allclose(mu_tk[live, D], widen(extra[0, :1])[0], rtol=1e-6)


def test_transformed_key_assignment_is_nearest_neighbour_in_d_plus_1():
    """The oracle's assignment on augmented rows is the exhaustive nearest neighbour between transformed
    keys and augmented centroids (brute force in d+1 dimensions), and it differs from the raw one when norms vary."""
    rng = np.random.default_rng(93)
    K = _rand_bits(rng, (1, 500, D), scale=1.0)
    K[0, ::3] = narrow(3.0 * widen(K[0, ::3]))                                        # mixed norms
    extra, _ = orc.key_extra_coordinate(K)
    Ka = orc.augment(K, extra)[0]
    mu = Ka[rng.choice(500, 12, replace=False)]
    a, best, _ = orc.assign(Ka, mu)
    kf, mf = widen(Ka).astype(np.float64), widen(mu).astype(np.float64)
    dist = ((kf[:, None, :] - mf[None, :, :]) ** 2).sum(-1)
    assert np.array_equal(a, dist.argmin(1).astype(np.int32))
    a_raw, _, _ = orc.assign(K[0], mu[:, :D].copy())
    assert (a != a_raw).sum() > 0


# ----------------------------------------------------------------------------- insertion on transformed keys
def _transformed_index(K, V, C, T, extra_tokens, seed, c2=None):
    """An oracle index built on the augmented rows [k, a(k)] (Lloyd in d+1 dims, pages of the d raw
    coordinates), with its geometry set for insertions.  K, V uint16 [U, n, D]."""
    U, n = K.shape[0], K.shape[1]
    rng = np.random.default_rng(seed)
    extra, c2 = orc.key_extra_coordinate(K, c2)
    Ka = orc.augment(K, extra)
    ix = orc.OracleIndex(U, 4, 16, C, max_tokens=n + extra_tokens)
    assign = np.empty((U, n), np.int32)
    cen_e, sum_e = np.zeros((U, C), np.float32), np.zeros((U, C), np.float32)
    for u in range(U):
        init = np.sort(rng.choice(n, C, replace=False)).astype(np.int32)
        a, mu, ssum, cnt, _ = orc.lloyd(Ka[u], init, T)
        assign[u] = a
        ix.centroid[u], ix.cluster_sum[u], ix.cluster_cnt[u] = mu[:, :D], ssum[:, :D], cnt
        cen_e[u], sum_e[u] = mu[:, D], ssum[:, D]
    ix.paginate(K, V, assign)
    key_extra = np.zeros((U, n + extra_tokens), np.uint16)
    key_extra[:, :n] = extra
    ix.set_geometry(c2.astype(np.float32), key_extra, cen_e, sum_e)
    return ix, assign


def test_transformed_insert_is_nearest_neighbour_in_d_plus_1_and_keeps_running_means():
    """Sec. 4.2 (last paragraph) with Eq. 2: the new key goes under its nearest centroid BETWEEN
    TRANSFORMED rows.  Brute force: direct ||[k, a] - [mu~, e~]||^2 over all clusters in d+1 dims.  The
    extra coordinate itself against its closed form, the a = 0 rule beyond the radius, and the
    running mean of the extra coordinate against the true mean of the members' coordinates."""
    rng = np.random.default_rng(101)
    U, n, C, steps = 2, 600, 9, 120
    K = _rand_bits(rng, (U, n + steps, D))
    K[:, ::3] = narrow(1.8 * widen(K[:, ::3]))                       # mixed norms: the coordinate matters
    V = _rand_bits(rng, (U, n + steps, D))
    ix, assign = _transformed_index(K[:, :n], V[:, :n], C, 3, steps, seed=5)
    members = [[list(np.nonzero(assign[u] == c)[0]) for c in range(C)] for u in range(U)]
    geo = ix.geometry
    c2 = geo["radius_sq"].astype(np.float64)
    differs_from_raw = 0
    for t in range(n, n + steps):
        k = K[:, t].copy()
        if t == n + 7:
            k = narrow(5.0 * widen(k))                                # longer than every prefill key
        mub = narrow(ix.centroid)
        eb = narrow(geo["centroid_extra"])
        chosen, best, second, extra = ix.insert(k, V[:, t])
        for u in range(U):
            kf = widen(k[u]).astype(np.float64)
            want = math.sqrt(max(c2[u] - (kf ** 2).sum(), 0.0))
            assert abs(float(widen(extra[u:u + 1])[0]) - want) <= 2.0 ** -8 * want
            if t == n + 7:
                assert extra[u] == 0
            assert geo["key_extra"][u, t] == extra[u]
            row = np.concatenate([kf, widen(extra[u:u + 1]).astype(np.float64)])
            cen = np.concatenate([widen(mub[u]).astype(np.float64), widen(eb[u]).astype(np.float64)[:, None]], 1)
            dist = ((row[None, :] - cen) ** 2).sum(1)
            assert chosen[u] == dist.argmin()
            np.testing.assert_allclose(best[u] + (row ** 2).sum(), dist.min(), atol=1e-9)
            raw = ((kf[None, :] - cen[:, :D]) ** 2).sum(1).argmin()
            differs_from_raw += int(raw != chosen[u])
            members[u][int(chosen[u])].append(t if t != n + 7 else -1)
    assert differs_from_raw > 0, "the extra coordinate never changed a decision: the case is vacuous"
    # running means = true means of the members, extra coordinate included
    Kall = K.copy()
    Kall[:, n + 7] = narrow(5.0 * widen(K[:, n + 7]))
    for u in range(U):
        for c in range(C):
            m = [x if x >= 0 else n + 7 for x in members[u][c]]
            assert ix.cluster_cnt[u, c] == len(m)
            if m:
                np.testing.assert_allclose(ix.centroid[u, c], widen(Kall[u, m]).astype(np.float64).mean(0), rtol=1e-5, atol=1e-5)
                np.testing.assert_allclose(geo["centroid_extra"][u, c], widen(geo["key_extra"][u, m]).astype(np.float64).mean(),
                                           rtol=1e-5, atol=1e-6)
                np.testing.assert_allclose(geo["cluster_sum_extra"][u, c], widen(geo["key_extra"][u, m]).astype(np.float64).sum(),
                                           rtol=1e-5, atol=1e-5)


def test_transformed_insert_with_equal_norms_is_the_raw_insert():
    """Keys in {+-1}^d all have squared norm d exactly, so with c^2 = d every extra coordinate is 0 and
    the transformed insertion must leave, bit for bit, the state the raw insertion leaves."""
    rng = np.random.default_rng(102)
    U, n, C, steps = 2, 300, 7, 60
    K = narrow((rng.integers(0, 2, (U, n + steps, D)) * 2 - 1).astype(np.float32))
    V = _rand_bits(rng, (U, n + steps, D))
    a_ix, assign = _transformed_index(K[:, :n], V[:, :n], C, 2, steps, seed=6)
    assert np.all(a_ix.geometry["key_extra"] == 0) and np.all(a_ix.geometry["radius_sq"] == D)
    b_ix = orc.OracleIndex(U, 4, 16, C, max_tokens=n + steps)
    b_ix.paginate(K[:, :n], V[:, :n], assign)
    b_ix.centroid[...], b_ix.cluster_sum[...], b_ix.cluster_cnt[...] = a_ix.centroid, a_ix.cluster_sum, a_ix.cluster_cnt
    for t in range(n, n + steps):
        ca = a_ix.insert(K[:, t], V[:, t])
        cb = b_ix.insert(K[:, t], V[:, t])
        assert np.array_equal(ca[0], cb[0]) and np.all(ca[3] == 0)
        np.testing.assert_allclose(ca[1], cb[1], atol=1e-12)
    for name in orc.OracleIndex.ARRAYS:
        assert np.array_equal(getattr(a_ix, name), getattr(b_ix, name)), name
    assert np.all(a_ix.geometry["centroid_extra"] == 0) and np.all(a_ix.geometry["cluster_sum_extra"] == 0)


def test_transformed_insert_override_and_force_are_followed():
    rng = np.random.default_rng(103)
    K = _rand_bits(rng, (1, 200, D))
    ix, _ = _transformed_index(K[:, :199], K[:, :199], 4, 1, 1, seed=7)
    before = ix.geometry["cluster_sum_extra"].copy()
    bits = int(narrow(np.array([2.5], np.float32))[0])
    chosen, _, _, own = ix.insert(K[:, 199], K[:, 199], force=np.array([3], np.int32), extra_override=np.array([bits], np.int32))
    assert chosen[0] == 3 and own[0] != bits
    assert ix.geometry["key_extra"][0, 199] == bits
    assert ix.geometry["cluster_sum_extra"][0, 3] == np.float32(before[0, 3] + np.float32(2.5))
    assert ix.geometry["centroid_extra"][0, 3] == np.float32(ix.geometry["cluster_sum_extra"][0, 3] / np.float32(ix.cluster_cnt[0, 3]))


# ----------------------------------------------------------------------------- three levels (Sec. 3.3, Alg. 4)
def _top_level(ix, C2, seed):
    """A top level over the clusters of an oracle index: Lloyd on the bf16-rounded centroids (the pinned
    routine), from C2 promoted clusters."""
    rng = np.random.default_rng(seed)
    top_c = np.zeros((ix.U, C2, D), np.float32)
    top_of = np.zeros((ix.U, ix.C), np.int32)
    for u in range(ix.U):
        init = np.sort(rng.choice(ix.C, C2, replace=False)).astype(np.int32)
        a, mu, _, _, _ = orc.lloyd(narrow(ix.centroid[u]), init, 3)
        top_c[u], top_of[u] = mu, a
    return top_c, top_of


@pytest.mark.parametrize("n_probe_top,n_probe,budget", [(3, 6, 128), (1, 4, 64), (5, 40, 256), (2, 2, 16)])
def test_three_level_select_is_the_staged_definition(n_probe_top, n_probe, budget):
    """numpy, stage by stage: best top nodes by the normalised GQA score of their bf16 rounding, best
    clusters among their children, best pages among those clusters' pages."""
    w = datagen.small(n_tokens=3000, n_clusters=40, n_kv_heads=3, n_components=24)
    ix, _, _ = _built(w)
    C2 = 8
    top_c, top_of = _top_level(ix, C2, 1)
    q = datagen.queries(w).reshape(ix.U, ix.G, D)
    ids, n_sel, scores, clusters, tops, Sc_all, St_all = ix.select_hier3(q, budget, n_probe_top, n_probe, top_c, top_of)
    qf = widen(q).astype(np.float64)
    S = _scores_numpy(ix, q)
    P = budget // ix.s
    for u in range(ix.U):
        nq = np.linalg.norm(qf[u], axis=1)
        st = np.float32(((widen(narrow(top_c[u])).astype(np.float64) @ qf[u].T) / nq[None]).max(1))
        np.testing.assert_allclose(St_all[u], st, rtol=1e-6)
        keep0 = sorted(sorted(range(C2), key=lambda t: (-St_all[u, t], t))[:n_probe_top])
        assert tops[u, :len(keep0)].tolist() == keep0 and np.all(tops[u, len(keep0):] == -1)
        sc = np.float32(((widen(narrow(ix.centroid[u])).astype(np.float64) @ qf[u].T) / nq[None]).max(1))
        np.testing.assert_allclose(Sc_all[u], sc, rtol=1e-6)
        children = [c for c in range(ix.C) if top_of[u, c] in keep0]
        keep1 = sorted(sorted(children, key=lambda c: (-Sc_all[u, c], c))[:n_probe])
        assert clusters[u, :len(keep1)].tolist() == keep1 and np.all(clusters[u, len(keep1):] == -1)
        cand = [p for p in range(ix.n_pages[u]) if ix.page_cluster[u, p] in keep1]
        want = sorted(sorted(cand, key=lambda p: (-S[u][p], p))[:P])
        assert n_sel[u] == len(want) and ids[u, :len(want)].tolist() == want


def test_three_level_select_with_every_top_node_is_the_two_level_select():
    w = datagen.small(n_tokens=3000, n_clusters=40, n_kv_heads=2, n_components=24)
    ix, _, _ = _built(w)
    top_c, top_of = _top_level(ix, 6, 2)
    q = datagen.queries(w).reshape(ix.U, ix.G, D)
    for n_refine in (0, 20):
        a = ix.select_hier3(q, 128, 6, 7, top_c, top_of, n_refine=n_refine)
        b = ix.select_hier(q, 128, 7, n_refine=n_refine)
        for x, y in zip(a[:4], b[:4]):
            assert np.array_equal(x, y)
    # one top node: only clusters hanging under it can be kept, only their pages returned
    ids, n_sel, _, clusters, tops, _, _ = ix.select_hier3(q, 16 * 500, 1, 40, top_c, top_of)
    for u in range(ix.U):
        t = tops[u, 0]
        kept = clusters[u][clusters[u] >= 0]
        assert set(kept.tolist()) == set(np.nonzero(top_of[u] == t)[0].tolist())
        got = ids[u, :n_sel[u]]
        assert set(ix.page_cluster[u, got].tolist()) <= set(kept.tolist())
        assert n_sel[u] == int(np.isin(ix.page_cluster[u, :ix.n_pages[u]], kept).sum())


# ----------------------------------------------------------------------------- change detector
def test_oracle_still_gives_the_stored_small_case():
    """tests/golden/oracle_small_case.json was written by tests/golden/write_oracle_fixture.py from the
    oracle alone; the oracle's answer on that seeded case must not drift unnoticed."""
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("write_oracle_fixture", os.path.join(here, "write_oracle_fixture.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = json.loads(json.dumps(mod.compute()))
    with open(os.path.join(here, "oracle_small_case.json")) as f:
        stored = json.load(f)
    for key in ("n_pages", "cluster_cnt", "insert_clusters", "page_ids", "n_selected", "sha256_16"):
        assert now[key] == stored[key], key
    for key in ("inertia", "scores", "out_head0_first8"):
        np.testing.assert_allclose(np.array(now[key]), np.array(stored[key]), rtol=1e-6, atol=1e-9)
