"""ctypes wrapper around the C oracle (oracle/ice_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, the smoke check and the benchmark's
cpu_baseline leg; never by the product package.  It allocates numpy arrays, passes their
pointers to the C functions and hands the arrays back.  The only arithmetic written here is
key_extra_coordinate (the extra coordinate of the transformed keys at prefill, Eq. 2, in numpy);
everything else is in the C file.  All state arrays carry a leading unit dimension
U = batch * n_kv_heads.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ice_oracle.c")
_LIB = os.path.join(_HERE, "libice_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add, OpenMP over units)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Geometry(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("radius_sq", "key_extra", "centroid_extra", "cluster_sum_extra")]


class _State(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("U", "d", "s", "C", "G", "max_pages", "max_tokens")] + \
               [(n, C.c_void_p) for n in ("n_tokens", "n_pages", "Kp", "Vp", "page_cluster", "page_fill",
                                          "page_pos", "cluster_tail", "cluster_cnt", "cluster_sum",
                                          "centroid", "page_sum", "rep")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_num_threads.restype = C.c_int
        _lib.orc_insert.restype = C.c_int
        _lib.orc_insert_transformed.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return lib().orc_num_threads()


def set_num_threads(t: int) -> None:
    lib().orc_set_num_threads(C.c_int(t))


def assign(K: np.ndarray, mu_bf16: np.ndarray):
    """Exhaustive nearest centroid for one unit.  K uint16 [n,d], mu_bf16 uint16 [C,d].
    Returns (a int32 [n], best float64 [n], second float64 [n])."""
    n, d = K.shape
    Cn = mu_bf16.shape[0]
    K = np.ascontiguousarray(K, np.uint16)
    mu_bf16 = np.ascontiguousarray(mu_bf16, np.uint16)
    a = np.empty(n, np.int32)
    best = np.empty(n, np.float64)
    second = np.empty(n, np.float64)
    lib().orc_assign(_p(K), _p(mu_bf16), C.c_int(n), C.c_int(Cn), C.c_int(d), _p(a), _p(best), _p(second))
    return a, best, second


def means(K: np.ndarray, a: np.ndarray, n_clusters: int, mu_prev: np.ndarray):
    """Means of the members for one unit; empty clusters keep mu_prev.  Returns (mu, sum, cnt)."""
    n, d = K.shape
    K = np.ascontiguousarray(K, np.uint16)
    a = np.ascontiguousarray(a, np.int32)
    mu = np.array(mu_prev, np.float32, copy=True, order="C")
    ssum = np.zeros((n_clusters, d), np.float32)
    cnt = np.zeros(n_clusters, np.int32)
    lib().orc_means(_p(K), _p(a), C.c_int(n), C.c_int(n_clusters), C.c_int(d), _p(mu), _p(ssum), _p(cnt))
    return mu, ssum, cnt


def lloyd(K: np.ndarray, init_idx: np.ndarray, T: int):
    """T Lloyd rounds for one unit from the promoted keys.  Returns (a, mu, sum, cnt, inertia[T])."""
    n, d = K.shape
    Cn = init_idx.shape[0]
    K = np.ascontiguousarray(K, np.uint16)
    init_idx = np.ascontiguousarray(init_idx, np.int32)
    a = np.empty(n, np.int32)
    mu = np.empty((Cn, d), np.float32)
    ssum = np.empty((Cn, d), np.float32)
    cnt = np.empty(Cn, np.int32)
    inertia = np.empty(T, np.float64)
    lib().orc_lloyd(_p(K), C.c_int(n), C.c_int(Cn), C.c_int(d), _p(init_idx), C.c_int(T),
                    _p(a), _p(mu), _p(ssum), _p(cnt), _p(inertia))
    return a, mu, ssum, cnt, inertia


class OracleIndex:
    """One layer's index for U units, as plain numpy arrays filled by the C oracle."""

    ARRAYS = ("n_tokens", "n_pages", "Kp", "Vp", "page_cluster", "page_fill", "page_pos",
              "cluster_tail", "cluster_cnt", "cluster_sum", "centroid", "page_sum", "rep")

    def __init__(self, U: int, group_size: int, page_size: int, n_clusters: int, max_tokens: int, d: int = 128,
                 max_pages: int | None = None, alloc_kv: bool = True):
        """max_pages overrides the default pool size (floor(max_tokens / page_size) + n_clusters), e.g. for
        an index that holds only a few gathered pages; alloc_kv=False leaves out the K/V page pools
        (selection needs only the representatives)."""
        self.U, self.G, self.s, self.C, self.d = U, group_size, page_size, n_clusters, d
        self.max_tokens = max_tokens
        self.max_pages = MP = max_tokens // page_size + n_clusters if max_pages is None else max_pages
        s, Cn = page_size, n_clusters
        self.n_tokens = np.zeros(U, np.int32)
        self.n_pages = np.zeros(U, np.int32)
        kv_pages = MP if alloc_kv else 1
        self.Kp = np.zeros((U, kv_pages, s, d), np.uint16)
        self.Vp = np.zeros((U, kv_pages, s, d), np.uint16)
        self.page_cluster = np.full((U, MP), -1, np.int32)
        self.page_fill = np.zeros((U, MP), np.int32)
        self.page_pos = np.full((U, MP, s), -1, np.int32)
        self.cluster_tail = np.full((U, Cn), -1, np.int32)
        self.cluster_cnt = np.zeros((U, Cn), np.int32)
        self.cluster_sum = np.zeros((U, Cn, d), np.float32)
        self.centroid = np.zeros((U, Cn, d), np.float32)
        self.page_sum = np.zeros((U, MP, d), np.float32)
        self.rep = np.zeros((U, MP, d), np.uint16)
        self.assign = None
        self.geometry = None

    def set_geometry(self, radius_sq, key_extra, centroid_extra, cluster_sum_extra):
        """Switches insertions to the transformed keys of Eq. 2.  radius_sq float32 [U] (c^2, fixed at
        prefill); key_extra uint16 [U, max_tokens] (a(k) of every token so far, by position);
        centroid_extra, cluster_sum_extra float32 [U, C] (mean and sum of the members' a).  Copies."""
        self.geometry = dict(
            radius_sq=np.array(radius_sq, np.float32, copy=True).reshape(self.U),
            key_extra=np.array(key_extra, np.uint16, copy=True).reshape(self.U, self.max_tokens),
            centroid_extra=np.array(centroid_extra, np.float32, copy=True).reshape(self.U, self.C),
            cluster_sum_extra=np.array(cluster_sum_extra, np.float32, copy=True).reshape(self.U, self.C))

    def _state(self) -> _State:
        st = _State()
        st.U, st.d, st.s, st.C, st.G = self.U, self.d, self.s, self.C, self.G
        st.max_pages, st.max_tokens = self.max_pages, self.max_tokens
        for name in self.ARRAYS:
            arr = getattr(self, name)
            assert arr.flags["C_CONTIGUOUS"]
            setattr(st, name, arr.ctypes.data)
        return st

    def _units(self, x: np.ndarray, tail: tuple, dtype) -> np.ndarray:
        x = np.ascontiguousarray(x, dtype).reshape((self.U,) + tail)
        return x

    def build(self, K: np.ndarray, V: np.ndarray, init_idx: np.ndarray, T: int):
        """K, V uint16 [..., n, d] (leading dims flatten to U); init_idx int32 [..., C]."""
        n = K.shape[-2]
        K = self._units(K, (n, self.d), np.uint16)
        V = self._units(V, (n, self.d), np.uint16)
        init_idx = self._units(init_idx, (self.C,), np.int32)
        self.assign = np.empty((self.U, n), np.int32)
        inertia = np.empty((self.U, T), np.float64)
        st = self._state()
        lib().orc_build(C.byref(st), _p(K), _p(V), C.c_int(n), _p(init_idx), C.c_int(T),
                        _p(self.assign), _p(inertia))
        return inertia

    def paginate(self, K: np.ndarray, V: np.ndarray, assign: np.ndarray):
        """Lay pages out for a given assignment (int32 [U, n]); cluster means are not touched."""
        n = K.shape[-2]
        K = self._units(K, (n, self.d), np.uint16)
        V = self._units(V, (n, self.d), np.uint16)
        assign = self._units(assign, (n,), np.int32)
        self.assign = assign.copy()
        st = self._state()
        lib().orc_paginate(C.byref(st), _p(K), _p(V), _p(assign), C.c_int(n))

    def insert(self, k: np.ndarray, v: np.ndarray, force: np.ndarray | None = None,
               extra_override: np.ndarray | None = None):
        """k, v uint16 [..., d].  Returns (chosen int32 [U], best float64 [U], second float64 [U]); after
        set_geometry the insertion is the one on the transformed keys and a fourth value is returned, the
        oracle's own extra coordinate of the new keys (uint16 [U]); extra_override int32 [U] (bf16 bits,
        -1 = none) then replaces it in everything that follows."""
        k = self._units(k, (self.d,), np.uint16)
        v = self._units(v, (self.d,), np.uint16)
        if force is not None:
            force = self._units(force, (), np.int32)
        chosen = np.empty(self.U, np.int32)
        best = np.empty(self.U, np.float64)
        second = np.empty(self.U, np.float64)
        st = self._state()
        if self.geometry is None:
            assert extra_override is None
            rc = lib().orc_insert(C.byref(st), _p(k), _p(v), _p(force), _p(chosen), _p(best), _p(second))
            if rc != 0:
                raise OverflowError("oracle insert: token capacity exceeded")
            return chosen, best, second
        geo = _Geometry()
        for name, arr in self.geometry.items():
            setattr(geo, name, arr.ctypes.data)
        if extra_override is not None:
            extra_override = self._units(extra_override, (), np.int32)
        extra = np.zeros(self.U, np.uint16)
        rc = lib().orc_insert_transformed(C.byref(st), C.byref(geo), _p(k), _p(v), _p(force), _p(extra_override),
                                          _p(chosen), _p(best), _p(second), _p(extra))
        if rc != 0:
            raise OverflowError("oracle insert: token capacity exceeded")
        return chosen, best, second, extra

    def select(self, q: np.ndarray, token_budget: int):
        """q uint16 [..., G, d] -> (ids int32 [U,P] ascending, -1 padded; n_sel [U]; scores [U,P];
        S_all float32 [U, max_pages])."""
        q = self._units(q, (self.G, self.d), np.uint16)
        P = token_budget // self.s
        ids = np.full((self.U, max(P, 1)), -1, np.int32)[:, :P].copy()
        n_sel = np.zeros(self.U, np.int32)
        scores = np.zeros((self.U, P), np.float32)
        S_all = np.full((self.U, self.max_pages), -np.inf, np.float32)
        st = self._state()
        lib().orc_select(C.byref(st), _p(q), C.c_int(token_budget), _p(ids), _p(n_sel), _p(scores), _p(S_all))
        return ids, n_sel, scores, S_all

    def select_hier(self, q: np.ndarray, token_budget: int, n_probe: int, n_refine: int = 0):
        """Staged selection: the n_probe best clusters by centroid score, then the best pages among
        theirs; with n_refine > 0 the n_refine best of those are re-ranked by their best key (needs the
        K tiles).  -> (ids int32 [U,P], n_sel [U], scores [U,P], clusters int32 [U,n_probe] ascending
        -1 padded, Sc_all float32 [U,C])."""
        q = self._units(q, (self.G, self.d), np.uint16)
        P = token_budget // self.s
        ids = np.full((self.U, P), -1, np.int32)
        n_sel = np.zeros(self.U, np.int32)
        scores = np.zeros((self.U, P), np.float32)
        clusters = np.full((self.U, n_probe), -1, np.int32)
        Sc_all = np.zeros((self.U, self.C), np.float32)
        st = self._state()
        lib().orc_select_hier(C.byref(st), _p(q), C.c_int(token_budget), C.c_int(n_probe), C.c_int(n_refine), _p(ids), _p(n_sel),
                              _p(scores), _p(clusters), _p(Sc_all))
        return ids, n_sel, scores, clusters, Sc_all

    def select_hier3(self, q: np.ndarray, token_budget: int, n_probe_top: int, n_probe: int, top_centroid: np.ndarray,
                     top_of: np.ndarray, n_refine: int = 0):
        """Three-level selection: the n_probe_top best top nodes (top_centroid float32 [U, C2, d]), then the
        n_probe best clusters among those hanging under them (top_of int32 [U, C]), then pages as
        select_hier.  -> (ids, n_sel, scores, clusters [U, n_probe], tops [U, n_probe_top], Sc_all [U, C],
        St_all [U, C2])."""
        q = self._units(q, (self.G, self.d), np.uint16)
        C2 = top_centroid.shape[-2]
        top_centroid = np.ascontiguousarray(top_centroid, np.float32).reshape(self.U, C2, self.d)
        top_of = np.ascontiguousarray(top_of, np.int32).reshape(self.U, self.C)
        P = token_budget // self.s
        ids = np.full((self.U, P), -1, np.int32)
        n_sel = np.zeros(self.U, np.int32)
        scores = np.zeros((self.U, P), np.float32)
        clusters = np.full((self.U, n_probe), -1, np.int32)
        tops = np.full((self.U, n_probe_top), -1, np.int32)
        Sc_all = np.zeros((self.U, self.C), np.float32)
        St_all = np.zeros((self.U, C2), np.float32)
        st = self._state()
        lib().orc_select_hier3(C.byref(st), _p(top_centroid), _p(top_of), C.c_int(C2), _p(q), C.c_int(token_budget),
                               C.c_int(n_probe_top), C.c_int(n_probe), C.c_int(n_refine), _p(ids), _p(n_sel), _p(scores),
                               _p(clusters), _p(tops), _p(Sc_all), _p(St_all))
        return ids, n_sel, scores, clusters, tops, Sc_all, St_all

    def attend(self, q: np.ndarray, ids: np.ndarray, n_sel: np.ndarray) -> np.ndarray:
        """Sparse attention over the listed pages: float32 [U, G, d]."""
        q = self._units(q, (self.G, self.d), np.uint16)
        P = ids.shape[-1]
        ids = self._units(ids, (P,), np.int32)
        n_sel = self._units(n_sel, (), np.int32)
        out = np.zeros((self.U, self.G, self.d), np.float32)
        st = self._state()
        lib().orc_attend(C.byref(st), _p(q), _p(ids), _p(n_sel), C.c_int(P), _p(out))
        return out

    def attend_resident(self, q: np.ndarray, ids: np.ndarray, n_sel: np.ndarray, rk: np.ndarray,
                        rv: np.ndarray) -> np.ndarray:
        """Attention over the listed pages and n_res resident tokens per unit (rk, rv uint16
        [..., n_res, d]) in one softmax: float32 [U, G, d]."""
        q = self._units(q, (self.G, self.d), np.uint16)
        P = ids.shape[-1]
        ids = self._units(ids, (P,), np.int32)
        n_sel = self._units(n_sel, (), np.int32)
        n_res = rk.shape[-2]
        rk = self._units(rk, (n_res, self.d), np.uint16)
        rv = self._units(rv, (n_res, self.d), np.uint16)
        out = np.zeros((self.U, self.G, self.d), np.float32)
        st = self._state()
        lib().orc_attend_resident(C.byref(st), _p(q), _p(ids), _p(n_sel), C.c_int(P), _p(rk), _p(rv),
                                  C.c_int(n_res), _p(out))
        return out

    def selected_tokens(self, ids: np.ndarray, n_sel: np.ndarray):
        """Sequence positions of the tokens of the listed pages: (pos int32 [U, P*s] -1 padded, n_tok [U])."""
        P = ids.shape[-1]
        ids = self._units(ids, (P,), np.int32)
        n_sel = self._units(n_sel, (), np.int32)
        pos = np.full((self.U, P * self.s), -1, np.int32)
        n_tok = np.zeros(self.U, np.int32)
        st = self._state()
        lib().orc_selected_tokens(C.byref(st), _p(ids), _p(n_sel), C.c_int(P), _p(pos), _p(n_tok))
        return pos, n_tok


def attend_tokens(q: np.ndarray, K: np.ndarray, V: np.ndarray, pos: np.ndarray, n_tok: np.ndarray) -> np.ndarray:
    """Attention over rows pos[u, :n_tok[u]] of a dense cache.  q uint16 [U, G, d]; K, V uint16
    [U, n_rows, d]; pos int32 [U, cap].  -> float32 [U, G, d]."""
    U, G, d = q.shape
    n_rows, cap = K.shape[1], pos.shape[1]
    q, K, V = (np.ascontiguousarray(a, np.uint16) for a in (q, K, V))
    pos, n_tok = np.ascontiguousarray(pos, np.int32), np.ascontiguousarray(n_tok, np.int32)
    out = np.zeros((U, G, d), np.float32)
    lib().orc_attend_tokens(_p(q), _p(K), _p(V), C.c_int(U), C.c_int(G), C.c_int(d), C.c_int(n_rows), _p(pos), _p(n_tok),
                            C.c_int(cap), _p(out))
    return out


# ---- transformed keys (Sec. 4.2, Eq. 2) -------------------------------------------------------------
def _bf16_rne(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def _bf16_to_f64(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def key_extra_coordinate(K: np.ndarray, c2: np.ndarray | None = None):
    """The one extra coordinate of c * T_K(k) = [k, sqrt(c^2 - ||k||^2)] for every key.
    K uint16 [U, n, d]; c2 float64 [U] or None (then c^2 = the largest squared key norm of the unit).
    Keys with ||k||^2 > c^2 get 0.  -> (extra uint16 [U, n] rounded to bf16, c2 float64 [U])."""
    n2 = (_bf16_to_f64(K) ** 2).sum(-1)
    if c2 is None:
        c2 = n2.max(-1)
    a = np.sqrt(np.maximum(np.asarray(c2, np.float64)[:, None] - n2, 0.0))
    return _bf16_rne(a.astype(np.float32)), np.asarray(c2, np.float64)


def augment(K: np.ndarray, extra: np.ndarray) -> np.ndarray:
    """[U, n, d] keys + [U, n] extra coordinate -> [U, n, d+1]: clustering on the transformed keys is
    clustering on these rows with the functions above (they take any d)."""
    return np.concatenate([np.ascontiguousarray(K, np.uint16), np.ascontiguousarray(extra, np.uint16)[..., None]], -1)
