"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

This module holds none of the method's arithmetic: it only draws keys, values,
queries and initial-centroid token indices with the shapes and value
distributions of the five benchmark workloads (Llama-3-8B-shaped GQA heads,
head_dim 128, keys from an isotropic Gaussian mixture) and rounds them once to
bf16 bit patterns (uint16).  Those same bits are handed to the CPU oracle and
to the HIP library, so neither side ever sees the other's output.

They stand in for the public long-context suites the paper evaluates on (their
items are not available and are never reproduced here); only the shapes are
taken from them.

Generator: numpy PCG64 seeded with the integer list [seed, sequence, head,
stream]; stream 0 = mixture centres, 1 = keys, 2 = values, 3 = queries,
4 = init indices, 5 = decode-loop draws.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

D = 128  # head_dim of every workload


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_kv_heads: int
    group_size: int          # query heads per KV head (GQA)
    n_tokens: int            # prefill context per (sequence, KV head)
    page_size: int
    n_clusters: int
    token_budget: int
    n_components: int        # Gaussians per head
    sigma: float             # per-coordinate std of a token around its centre
    value_kind: str          # "mixture" or "normal"
    outlier_frac: float = 0.0
    decode_steps: int = 0    # > 0: long-generation loop
    drift: float = 0.0       # per-step, per-coordinate std of the centre drift
    seed: int = 1
    n_super: int = 0         # > 0: nested mixture, the centres themselves gather around n_super points
    super_spread: float = 0.0  # per-coordinate std of a centre around its point


# The five workloads of the benchmark definition.  n_clusters of configs 4 and 5
# is not restated there; n_tokens / 64 is used, as in configs 2 and 3.
WORKLOADS = {
    "cfg1": Workload("cfg1", 1, 2, 4, 4096, 16, 32, 256, 32, 0.3, "mixture", seed=1),
    "cfg2": Workload("cfg2", 1, 8, 4, 32768, 16, 512, 256, 256, 0.3, "normal", seed=1000),
    "cfg3": Workload("cfg3", 1, 8, 4, 131072, 16, 2048, 1024, 1024, 0.3, "normal",
                     outlier_frac=0.05, seed=3000),
    "cfg4": Workload("cfg4", 16, 8, 4, 32768, 16, 512, 256, 256, 0.3, "normal", seed=4000),
    "cfg5": Workload("cfg5", 1, 8, 4, 16384, 16, 256, 256, 256, 0.3, "normal",
                     decode_steps=4096, drift=0.01, seed=5000),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, seq: int, head: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, seq, head, stream]))


def centres(w: Workload, seed: int | None = None) -> np.ndarray:
    """Mixture centres ~ N(0, I): float32 [batch, n_kv_heads, n_components, D]."""
    seed = w.seed if seed is None else seed
    out = np.empty((w.batch, w.n_kv_heads, w.n_components, D), dtype=np.float32)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            r = _rng(seed, b, h, 0)
            if w.n_super > 0:   # structure above the centres: what a level above the clusters can summarise
                sup = r.standard_normal((w.n_super, D), dtype=np.float32)
                out[b, h] = sup[r.integers(0, w.n_super, size=w.n_components)] + np.float32(w.super_spread) * r.standard_normal(
                    (w.n_components, D), dtype=np.float32)
            else:
                out[b, h] = r.standard_normal((w.n_components, D), dtype=np.float32)
    return out


def _mixture_rows(rng, cen, n, sigma):
    comp = rng.integers(0, cen.shape[0], size=n)
    x = rng.standard_normal((n, D), dtype=np.float32)
    x *= np.float32(sigma)
    x += cen[comp]
    return x


def _map_units(fn, w: Workload, workers: int):
    """fn(b, h) for every (sequence, KV head); with workers > 1 on a thread pool (every unit draws from a
    generator of its own, so the result does not depend on the schedule)."""
    units = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    if workers <= 1 or len(units) == 1:
        for b, h in units:
            fn(b, h)
        return
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(workers, len(units))) as ex:
        list(ex.map(lambda bh: fn(*bh), units))


def keys_values(w: Workload, seed: int | None = None, n_tokens: int | None = None, workers: int = 1):
    """Prefill keys and values as bf16 bits: two uint16 arrays [batch, n_kv_heads, n, D]."""
    seed = w.seed if seed is None else seed
    n = w.n_tokens if n_tokens is None else n_tokens
    cen = centres(w, seed)
    K = np.empty((w.batch, w.n_kv_heads, n, D), dtype=np.uint16)
    V = np.empty_like(K)

    def one(b, h):
        rk = _rng(seed, b, h, 1)
        x = _mixture_rows(rk, cen[b, h], n, w.sigma)
        if w.outlier_frac > 0.0:
            m = rk.random(n) < w.outlier_frac
            x[m] = rk.uniform(-3.0, 3.0, size=(int(m.sum()), D)).astype(np.float32)
        K[b, h] = f32_to_bf16_bits(x)
        rv = _rng(seed, b, h, 2)
        if w.value_kind == "mixture":
            vc = rv.standard_normal((w.n_components, D), dtype=np.float32)
            y = _mixture_rows(rv, vc, n, w.sigma)
        else:
            y = rv.standard_normal((n, D), dtype=np.float32)
        V[b, h] = f32_to_bf16_bits(y)

    _map_units(one, w, workers)
    return K, V


def queries(w: Workload, seed: int | None = None, step: int = 0, cen: np.ndarray | None = None) -> np.ndarray:
    """One decode query per query head: random centre of its KV head + sigma*N(0, I).

    Returns bf16 bits, uint16 [batch, n_kv_heads * group_size, D]; query head
    h_q belongs to KV head h_q // group_size.
    """
    seed = w.seed if seed is None else seed
    cen = centres(w, seed) if cen is None else cen
    q = np.empty((w.batch, w.n_kv_heads * w.group_size, D), dtype=np.uint16)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            r = _rng(seed, b, h, 3 + 16 * (step + 1))
            x = _mixture_rows(r, cen[b, h], w.group_size, w.sigma)
            q[b, h * w.group_size:(h + 1) * w.group_size] = f32_to_bf16_bits(x)
    return q


def init_indices(w: Workload, seed: int | None = None, n_tokens: int | None = None) -> np.ndarray:
    """n_clusters distinct token indices per unit (the promoted keys): int32 [batch, n_kv_heads, C]."""
    seed = w.seed if seed is None else seed
    n = w.n_tokens if n_tokens is None else n_tokens
    out = np.empty((w.batch, w.n_kv_heads, w.n_clusters), dtype=np.int32)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            out[b, h] = np.sort(_rng(seed, b, h, 4).choice(n, size=w.n_clusters, replace=False))
    return out


class DecodeStream:
    """Long-generation inputs: each step drifts every centre by N(0, drift^2 I), then draws one
    new key (random centre + sigma*N), one N(0,1) value and one query per query head."""

    def __init__(self, w: Workload, seed: int | None = None):
        self.w = w
        self.seed = w.seed if seed is None else seed
        self.cen = centres(w, self.seed).copy()
        self.step = 0

    def _unit_step(self, b, h, step, k_out, v_out, q_out):
        """One step of one (sequence, KV head): drift, new key and value, the group's queries."""
        w = self.w
        r = _rng(self.seed, b, h, 5 + 16 * (step + 1))
        self.cen[b, h] += np.float32(w.drift) * r.standard_normal(self.cen[b, h].shape, dtype=np.float32)
        k_out[b, h] = f32_to_bf16_bits(_mixture_rows(r, self.cen[b, h], 1, w.sigma)[0])
        v_out[b, h] = f32_to_bf16_bits(r.standard_normal(D, dtype=np.float32))
        rq = _rng(self.seed, b, h, 3 + 16 * (step + 2))
        q_out[b, h * w.group_size:(h + 1) * w.group_size] = f32_to_bf16_bits(_mixture_rows(rq, self.cen[b, h], w.group_size, w.sigma))

    def next(self):
        w = self.w
        k = np.empty((w.batch, w.n_kv_heads, D), dtype=np.uint16)
        v = np.empty_like(k)
        q = np.empty((w.batch, w.n_kv_heads * w.group_size, D), dtype=np.uint16)
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                self._unit_step(b, h, self.step, k, v, q)
        self.step += 1
        return k, v, q

    def take(self, m: int, workers: int = 1):
        """The next m steps at once: k, v uint16 [m, batch, n_kv_heads, D], q uint16 [m, batch, H_q, D]; the
        same values m calls of next() give.  Units are independent; with workers > 1 they are spread
        over forked processes (call it before the process initialises a GPU)."""
        w = self.w
        k = np.empty((m, w.batch, w.n_kv_heads, D), dtype=np.uint16)
        v = np.empty_like(k)
        q = np.empty((m, w.batch, w.n_kv_heads * w.group_size, D), dtype=np.uint16)
        units = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
        if workers > 1 and len(units) > 1:
            import multiprocessing
            with multiprocessing.get_context("fork").Pool(min(workers, len(units))) as pool:
                parts = pool.map(_stream_unit, [(self, b, h, m) for b, h in units])
        else:
            parts = [_stream_unit((self, b, h, m)) for b, h in units]
        G = w.group_size
        for (b, h), (ku, vu, qu, cen) in zip(units, parts):
            k[:, b, h], v[:, b, h], q[:, b, h * G:(h + 1) * G] = ku, vu, qu
            self.cen[b, h] = cen
        self.step += m
        return k, v, q


def _stream_unit(args):
    """m steps of one (sequence, KV head) of a DecodeStream: (k [m, D], v [m, D], q [m, G, D], centres after)."""
    st, b, h, m = args
    w = st.w
    k = np.empty((m, w.batch, w.n_kv_heads, D), dtype=np.uint16)
    v = np.empty_like(k)
    q = np.empty((m, w.batch, w.n_kv_heads * w.group_size, D), dtype=np.uint16)
    for t in range(m):
        st._unit_step(b, h, st.step + t, k[t], v[t], q[t])
    G = w.group_size
    return k[:, b, h].copy(), v[:, b, h].copy(), q[:, b, h * G:(h + 1) * G].copy(), st.cen[b, h]


def small(name: str = "tiny", **kw) -> Workload:
    """A reduced workload with the same recipe, for tests (sizes are keyword-overridable)."""
    base = dict(name=name, batch=1, n_kv_heads=2, group_size=4, n_tokens=1000, page_size=16,
                n_clusters=24, token_budget=128, n_components=16, sigma=0.3,
                value_kind="normal", seed=7)
    base.update(kw)
    return Workload(**base)
