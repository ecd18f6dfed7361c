"""GPU test of ice_attend_noalloc, the attention entry point whose scratch (the partial sums of the
page list's shares) is a static device array of the library instead of a workspace region: through
the C ABI, against ice_attend on the same index, queries and page lists, on calls in a row that
shrink (the array keeps the previous call's contents), and against the CPU oracle."""
import numpy as np
import pytest
import torch

import datagen
from tests.util import D, down, export_np, oracle_from_export, up

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3        # contract: max-abs on bf16 inputs with fp32 accumulation
ATTN_EXPECTED = 2e-4   # regression guard (both sides accumulate in fp32)


def _index(n_kv_heads, n_tokens, n_clusters, seed):
    from paper_2604_10539_amd import IceIndex
    w = datagen.small(n_tokens=n_tokens, n_clusters=n_clusters, n_kv_heads=n_kv_heads, n_components=n_clusters, seed=seed)
    K, V = datagen.keys_values(w)
    ix = IceIndex(w.batch, w.n_kv_heads, w.group_size, w.n_tokens, w.page_size, w.n_clusters, kmeans_iters=2,
                  init_idx=up(datagen.init_indices(w)))
    ix.build_index(up(K), up(V))
    return w, ix


def _both(ix, q, ids, n_sel):
    from paper_2604_10539_amd import binding as b
    P = int(ids.shape[-1])
    ref = torch.full((ix.batch, ix.n_kv_heads * ix.group_size, D), 7.0, dtype=torch.float32, device="cuda")
    got = torch.full_like(ref, -7.0)
    b.ice_attend(ix.handle, q, ids, n_sel, P, ref)
    b.ice_attend_noalloc(ix.handle, q, ids, n_sel, P, got)
    torch.cuda.synchronize()
    return down(ref), down(got)


def test_noalloc_attention_equals_ice_attend_on_shrinking_calls():
    w, ix = _index(2, 6000, 40, seed=21)
    ex = export_np(ix)
    o = oracle_from_export(ix, ex)
    # three calls in a row on one GPU: 96 pages per unit (6 shares), then 20 (2 shares), then 3 (1 share);
    # every later call leaves most of the array as the call before wrote it
    for step, budget in enumerate((96 * 16, 20 * 16, 3 * 16)):
        qn = datagen.queries(w, step=step)
        q = up(qn)
        ids, n_sel, _ = ix.select(q, budget)
        ref, got = _both(ix, q, ids, n_sel)
        err = np.abs(got - ref).max()
        exp = o.attend(qn, down(ids).reshape(ix.U, -1), down(n_sel).reshape(ix.U)).reshape(ref.shape)
        err_o = np.abs(got - exp).max()
        print("[noalloc] budget %d: vs ice_attend %.2e, vs oracle %.2e" % (budget, err, err_o))
        assert err <= ATTN_EXPECTED and err <= ATTN_TOL
        assert err_o <= ATTN_EXPECTED and err_o <= ATTN_TOL
    # a smaller index afterwards (other unit count, other page count), then a unit with an empty list
    w2, ix2 = _index(1, 1500, 24, seed=22)
    q2 = up(datagen.queries(w2))
    ids2, n_sel2, _ = ix2.select(q2, 8 * 16)
    ref, got = _both(ix2, q2, ids2, n_sel2)
    assert np.abs(got - ref).max() <= ATTN_EXPECTED
    n0 = torch.zeros_like(n_sel2)
    ref, got = _both(ix2, q2, ids2, n0)
    assert np.array_equal(ref, np.zeros_like(ref)) and np.array_equal(got, ref)


def test_noalloc_attention_rejects_more_units_than_the_array_holds():
    from paper_2604_10539_amd import IceIndex, binding as b
    w = datagen.small(n_tokens=64, n_clusters=2, n_kv_heads=257, n_components=2)
    K, V = datagen.keys_values(w)
    ix = IceIndex(1, 257, 4, 64, 16, 2, kmeans_iters=1)
    ix.build_index(up(K), up(V))
    q = up(datagen.queries(w))
    ids, n_sel, _ = ix.select(q, 32)
    out = torch.zeros((1, 257 * 4, D), dtype=torch.float32, device="cuda")
    with pytest.raises(b.IceError) as e:
        b.ice_attend_noalloc(ix.handle, q, ids, n_sel, int(ids.shape[-1]), out)
    assert e.value.status == b.ICE_ERR_UNSUPPORTED and "256" in str(e.value)
    torch.cuda.synchronize()
