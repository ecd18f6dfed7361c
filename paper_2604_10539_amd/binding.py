"""Thin ctypes binding of the C ABI in include/icecache.h (same names, argument marshalling only).

Every step of the path runs in the HIP library; torch supplies device memory and the current
stream.  There is no fallback: if libicecache.so is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libicecache.so")

ICE_OK, ICE_ERR_INVALID_ARG, ICE_ERR_SHAPE, ICE_ERR_STATE, ICE_ERR_CAPACITY, ICE_ERR_UNSUPPORTED, ICE_ERR_DEVICE = range(7)
STATUS_NAMES = ["ICE_OK", "ICE_ERR_INVALID_ARG", "ICE_ERR_SHAPE", "ICE_ERR_STATE", "ICE_ERR_CAPACITY",
                "ICE_ERR_UNSUPPORTED", "ICE_ERR_DEVICE"]
SYMBOLS = ["ice_workspace_bytes", "ice_create", "ice_destroy", "ice_build_index", "ice_insert", "ice_insert_batch", "ice_select",
           "ice_attend", "ice_attend_noalloc", "ice_select_attend", "ice_attend_resident", "ice_select_attend_resident", "ice_selected_tokens", "ice_attend_tokens", "ice_select_hier", "ice_select_hier3", "ice_build_top_level", "ice_export_top_level", "ice_set_geometry", "ice_export_geometry", "ice_export_index", "ice_import_index", "ice_debug_assign", "ice_debug_rerun_stage", "ice_debug_select_fault",
           "ice_debug_peak_read", "ice_debug_peak_mfma", "ice_last_error"]


class IceConfig(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_kv_heads", C.c_int32), ("group_size", C.c_int32), ("head_dim", C.c_int32),
                ("max_tokens", C.c_int32), ("kmeans_iters", C.c_int32), ("seed", C.c_uint64),
                ("init_idx", C.c_void_p)]


class IceIndexView(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_units", "group_size", "head_dim", "page_size", "n_clusters", "cpad",
                                         "max_pages", "max_tokens", "n_tokens", "reserved")] + \
               [(n, C.c_void_p) for n in ("Kp", "Vp", "page_cluster", "page_fill", "page_pos", "cluster_tail",
                                          "cluster_cnt", "cluster_sum", "centroid", "page_sum", "rep", "n_pages",
                                          "assign", "assign_centroid_bf16", "init_idx")]


class IceTopView(C.Structure):
    _fields_ = [("n_top", C.c_int32), ("n_top_max", C.c_int32), ("top_centroid", C.c_void_p), ("top_centroid_bf16", C.c_void_p),
                ("top_of", C.c_void_p), ("top_count", C.c_void_p), ("top_init", C.c_void_p)]


class IceGeometryView(C.Structure):
    _fields_ = [("geometry", C.c_int32), ("reserved", C.c_int32), ("key_extra", C.c_void_p),
                ("centroid_extra", C.c_void_p), ("cluster_sum_extra", C.c_void_p), ("radius_sq", C.c_void_p),
                ("assign_centroid_extra_bf16", C.c_void_p)]


ICE_GEOMETRY_RAW, ICE_GEOMETRY_TRANSFORMED = 0, 1


class IceError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < 7 else status, message))
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Loads the HIP library built by paper_2604_10539_amd/build.py; raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no fallback path)" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        L.ice_last_error.restype = C.c_char_p
        L.ice_workspace_bytes.restype = C.c_size_t
        L.ice_workspace_bytes.argtypes = [C.POINTER(IceConfig), C.c_int32, C.c_int32]
        L.ice_create.argtypes = [C.POINTER(IceConfig), C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)]
        L.ice_destroy.argtypes = [C.c_void_p]
        L.ice_build_index.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.ice_insert.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ice_insert_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.ice_select.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ice_attend.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.ice_attend_noalloc.argtypes = L.ice_attend.argtypes
        L.ice_select_attend.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p]
        L.ice_attend_resident.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                          C.c_int32, C.c_void_p, C.c_void_p]
        L.ice_select_attend_resident.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ice_selected_tokens.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ice_attend_tokens.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                        C.c_int32, C.c_void_p, C.c_void_p]
        L.ice_select_hier.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ice_select_hier3.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ice_build_top_level.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.ice_export_top_level.argtypes = [C.c_void_p, C.POINTER(IceTopView)]
        L.ice_set_geometry.argtypes = [C.c_void_p, C.c_int32]
        L.ice_export_geometry.argtypes = [C.c_void_p, C.POINTER(IceGeometryView)]
        L.ice_export_index.argtypes = [C.c_void_p, C.POINTER(IceIndexView)]
        L.ice_import_index.argtypes = [C.c_void_p, C.POINTER(IceIndexView), C.c_void_p]
        L.ice_debug_assign.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_void_p]
        L.ice_debug_rerun_stage.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.ice_debug_select_fault.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                             C.c_int32, C.c_void_p]
        L.ice_debug_peak_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.ice_debug_peak_mfma.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.c_void_p]
        for name in SYMBOLS:
            if name not in ("ice_last_error", "ice_workspace_bytes"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def ice_last_error() -> str:
    return lib().ice_last_error().decode()


def _check(status: int) -> None:
    if status != ICE_OK:
        raise IceError(status, ice_last_error())


def _ptr(t) -> int | None:
    """Device (or any) address of a tensor; None stays NULL; ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors handed to the library must be contiguous"
    return t.data_ptr()


def _stream(stream) -> int | None:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return stream if isinstance(stream, int) else stream.cuda_stream


def make_config(batch, n_kv_heads, group_size, max_tokens, kmeans_iters=10, seed=0, init_idx=None, head_dim=128):
    return IceConfig(batch, n_kv_heads, group_size, head_dim, max_tokens, kmeans_iters, seed, _ptr(init_idx))


def ice_workspace_bytes(cfg: IceConfig, page_size: int, n_clusters: int) -> int:
    return lib().ice_workspace_bytes(C.byref(cfg), page_size, n_clusters)


def ice_create(cfg: IceConfig, workspace, workspace_bytes: int | None = None) -> int:
    """workspace: a uint8 device tensor (or a raw address together with workspace_bytes)."""
    out = C.c_void_p()
    nbytes = workspace_bytes if workspace_bytes is not None else workspace.numel() * workspace.element_size()
    _check(lib().ice_create(C.byref(cfg), _ptr(workspace), nbytes, C.byref(out)))
    return out.value


def ice_destroy(idx: int) -> None:
    _check(lib().ice_destroy(idx))


def ice_build_index(idx, K, V, n_tokens, page_size, n_clusters, stream=None) -> None:
    _check(lib().ice_build_index(idx, _ptr(K), _ptr(V), n_tokens, page_size, n_clusters, _stream(stream)))


def ice_insert(idx, k, v, stream=None) -> None:
    _check(lib().ice_insert(idx, _ptr(k), _ptr(v), _stream(stream)))


def ice_insert_batch(idx, k, v, m, stream=None) -> None:
    _check(lib().ice_insert_batch(idx, _ptr(k), _ptr(v), m, _stream(stream)))


def ice_select(idx, q, token_budget, page_ids, n_selected, scores=None, stream=None) -> None:
    _check(lib().ice_select(idx, _ptr(q), token_budget, _ptr(page_ids), _ptr(n_selected), _ptr(scores), _stream(stream)))


def ice_attend(idx, q, page_ids, n_selected, n_ids_per_unit, out, stream=None) -> None:
    _check(lib().ice_attend(idx, _ptr(q), _ptr(page_ids), _ptr(n_selected), n_ids_per_unit, _ptr(out), _stream(stream)))


def ice_attend_noalloc(idx, q, page_ids, n_selected, n_ids_per_unit, out, stream=None) -> None:
    _check(lib().ice_attend_noalloc(idx, _ptr(q), _ptr(page_ids), _ptr(n_selected), n_ids_per_unit, _ptr(out),
                                    _stream(stream)))


def ice_select_attend(idx, q, token_budget, page_ids, n_selected, out, stream=None) -> None:
    _check(lib().ice_select_attend(idx, _ptr(q), token_budget, _ptr(page_ids), _ptr(n_selected), _ptr(out),
                                   _stream(stream)))


def ice_attend_resident(idx, q, page_ids, n_selected, n_ids_per_unit, resident_k, resident_v, n_resident, out,
                        stream=None) -> None:
    _check(lib().ice_attend_resident(idx, _ptr(q), _ptr(page_ids), _ptr(n_selected), n_ids_per_unit, _ptr(resident_k),
                                     _ptr(resident_v), n_resident, _ptr(out), _stream(stream)))


def ice_select_attend_resident(idx, q, token_budget, resident_k, resident_v, n_resident, page_ids, n_selected, out,
                               stream=None) -> None:
    _check(lib().ice_select_attend_resident(idx, _ptr(q), token_budget, _ptr(resident_k), _ptr(resident_v), n_resident,
                                            _ptr(page_ids), _ptr(n_selected), _ptr(out), _stream(stream)))


def ice_selected_tokens(idx, page_ids, n_selected, n_ids_per_unit, token_pos, n_tok, stream=None) -> None:
    _check(lib().ice_selected_tokens(idx, _ptr(page_ids), _ptr(n_selected), n_ids_per_unit, _ptr(token_pos), _ptr(n_tok),
                                     _stream(stream)))


def ice_attend_tokens(idx, q, K, V, n_rows, token_pos, n_tok, max_tok, out, stream=None) -> None:
    _check(lib().ice_attend_tokens(idx, _ptr(q), _ptr(K), _ptr(V), n_rows, _ptr(token_pos), _ptr(n_tok), max_tok,
                                   _ptr(out), _stream(stream)))


def ice_select_hier(idx, q, token_budget, n_probe, page_ids, n_selected, scores=None, clusters=None, out=None,
                    stream=None, n_refine=0) -> None:
    _check(lib().ice_select_hier(idx, _ptr(q), token_budget, n_probe, n_refine, _ptr(page_ids), _ptr(n_selected), _ptr(scores),
                                 _ptr(clusters), _ptr(out), _stream(stream)))


def ice_select_hier3(idx, q, token_budget, n_probe_top, n_probe, page_ids, n_selected, scores=None, clusters=None, tops=None,
                     out=None, stream=None, n_refine=0) -> None:
    _check(lib().ice_select_hier3(idx, _ptr(q), token_budget, n_probe_top, n_probe, n_refine, _ptr(page_ids), _ptr(n_selected),
                                  _ptr(scores), _ptr(clusters), _ptr(tops), _ptr(out), _stream(stream)))


def ice_build_top_level(idx, n_top: int, iters: int, stream=None) -> None:
    _check(lib().ice_build_top_level(idx, n_top, iters, _stream(stream)))


def ice_export_top_level(idx) -> IceTopView:
    view = IceTopView()
    _check(lib().ice_export_top_level(idx, C.byref(view)))
    return view


def ice_set_geometry(idx, geometry: int) -> None:
    _check(lib().ice_set_geometry(idx, geometry))


def ice_export_geometry(idx) -> IceGeometryView:
    view = IceGeometryView()
    _check(lib().ice_export_geometry(idx, C.byref(view)))
    return view


def ice_export_index(idx) -> IceIndexView:
    view = IceIndexView()
    _check(lib().ice_export_index(idx, C.byref(view)))
    return view


def ice_import_index(idx, view: IceIndexView, stream=None) -> None:
    _check(lib().ice_import_index(idx, C.byref(view), _stream(stream)))


def ice_debug_assign(idx, K, n, centroids_bf16, n_clusters, assign_out, best_out=None, stream=None) -> None:
    _check(lib().ice_debug_assign(idx, _ptr(K), n, _ptr(centroids_bf16), n_clusters, _ptr(assign_out),
                                  _ptr(best_out), _stream(stream)))


ICE_STAGE_ASSIGN, ICE_STAGE_SORT, ICE_STAGE_MEANS, ICE_STAGE_PAGINATE = range(4)


def ice_debug_rerun_stage(idx, K, V, stage, stream=None) -> None:
    _check(lib().ice_debug_rerun_stage(idx, _ptr(K), _ptr(V), stage, _stream(stream)))


def ice_debug_select_fault(idx, q, token_budget, page_ids, n_selected, out, muted_chunk, wait_log2, stream=None) -> None:
    _check(lib().ice_debug_select_fault(idx, _ptr(q), token_budget, _ptr(page_ids), _ptr(n_selected), _ptr(out), muted_chunk,
                                        wait_log2, _stream(stream)))


def ice_debug_peak_read(buf, nbytes, sink, stream=None) -> None:
    _check(lib().ice_debug_peak_read(_ptr(buf), nbytes, _ptr(sink), _stream(stream)))


def ice_debug_peak_mfma(sink, iters, stream=None) -> float:
    """Enqueues the MFMA loop; returns the flop count of the launch."""
    flops = C.c_double(0.0)
    _check(lib().ice_debug_peak_mfma(_ptr(sink), iters, C.byref(flops), _stream(stream)))
    return flops.value


# ------------------------------------------------------------------------------------------------
_VIEW_FIELDS = {  # name -> (torch dtype, shape as a function of the view)
    "Kp": (torch.int16, lambda v: (v.n_units, v.max_pages, v.page_size, v.head_dim)),
    "Vp": (torch.int16, lambda v: (v.n_units, v.max_pages, v.page_size, v.head_dim)),
    "page_cluster": (torch.int32, lambda v: (v.n_units, v.max_pages)),
    "page_fill": (torch.int32, lambda v: (v.n_units, v.max_pages)),
    "page_pos": (torch.int32, lambda v: (v.n_units, v.max_pages, v.page_size)),
    "cluster_tail": (torch.int32, lambda v: (v.n_units, v.n_clusters)),
    "cluster_cnt": (torch.int32, lambda v: (v.n_units, v.n_clusters)),
    "cluster_sum": (torch.float32, lambda v: (v.n_units, v.n_clusters, v.head_dim)),
    "centroid": (torch.float32, lambda v: (v.n_units, v.n_clusters, v.head_dim)),
    "page_sum": (torch.float32, lambda v: (v.n_units, v.max_pages, v.head_dim)),
    "rep": (torch.int16, lambda v: (v.n_units, v.max_pages, v.head_dim)),
    "n_pages": (torch.int32, lambda v: (v.n_units,)),
    "assign": (torch.int32, lambda v: (v.n_units, v.max_tokens)),
    "assign_centroid_bf16": (torch.int16, lambda v: (v.n_units, v.cpad, v.head_dim)),
    "init_idx": (torch.int32, lambda v: (v.n_units, v.n_clusters)),
}
IMPORT_FIELDS = ("Kp", "Vp", "page_cluster", "page_fill", "page_pos", "cluster_tail", "cluster_cnt", "cluster_sum",
                 "centroid", "page_sum", "rep", "n_pages")


class IceIndex:
    """Owns the workspace tensor and the index handle; every method is one C-ABI call.
    bf16 tensors may be torch.bfloat16 or int16 bit patterns."""

    def __init__(self, batch, n_kv_heads, group_size, max_tokens, page_size, n_clusters, kmeans_iters=10, seed=0,
                 init_idx=None, device="cuda", geometry=ICE_GEOMETRY_RAW):
        self.batch, self.n_kv_heads, self.group_size = batch, n_kv_heads, group_size
        self.page_size, self.n_clusters, self.max_tokens = page_size, n_clusters, max_tokens
        self.U = batch * n_kv_heads
        self.device = torch.device(device)
        self._init_idx = init_idx  # keeps the device tensor alive: the library reads it at build time
        self.cfg = make_config(batch, n_kv_heads, group_size, max_tokens, kmeans_iters, seed, init_idx)
        nbytes = ice_workspace_bytes(self.cfg, page_size, n_clusters)
        if nbytes == 0:
            raise IceError(ICE_ERR_INVALID_ARG, "invalid configuration")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.handle = ice_create(self.cfg, self.workspace)
        if geometry != ICE_GEOMETRY_RAW:
            ice_set_geometry(self.handle, geometry)

    def close(self):
        if getattr(self, "handle", None):
            ice_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def build_index(self, K, V, stream=None):
        n = K.shape[-2]
        ice_build_index(self.handle, K, V, n, self.page_size, self.n_clusters, stream)

    def insert(self, k, v, stream=None):
        ice_insert(self.handle, k, v, stream)

    def insert_batch(self, k, v, stream=None):
        """k, v: [B, H_kv, m, 128]; the m tokens are inserted in order, as m insert() calls would."""
        ice_insert_batch(self.handle, k, v, int(k.shape[-2]), stream)

    def _sel_buffers(self, token_budget):
        P = max(token_budget // self.page_size, 1)
        ids = torch.empty((self.batch, self.n_kv_heads, P), dtype=torch.int32, device=self.device)
        n_sel = torch.empty((self.batch, self.n_kv_heads), dtype=torch.int32, device=self.device)
        return ids, n_sel

    def select(self, q, token_budget, with_scores=True, stream=None):
        ids, n_sel = self._sel_buffers(token_budget)
        scores = torch.empty(ids.shape, dtype=torch.float32, device=self.device) if with_scores else None
        ice_select(self.handle, q, token_budget, ids, n_sel, scores, stream)
        return ids, n_sel, scores

    def attend(self, q, page_ids, n_selected, out=None, stream=None):
        if out is None:
            out = torch.empty((self.batch, self.n_kv_heads * self.group_size, 128), dtype=torch.float32,
                              device=self.device)
        ice_attend(self.handle, q, page_ids, n_selected, page_ids.shape[-1], out, stream)
        return out

    def select_attend(self, q, token_budget, ids=None, n_sel=None, out=None, stream=None):
        if ids is None:
            ids, n_sel = self._sel_buffers(token_budget)
        if out is None:
            out = torch.empty((self.batch, self.n_kv_heads * self.group_size, 128), dtype=torch.float32,
                              device=self.device)
        ice_select_attend(self.handle, q, token_budget, ids, n_sel, out, stream)
        return ids, n_sel, out

    def attend_resident(self, q, ids, n_sel, resident_k, resident_v, out=None, stream=None):
        """resident_k, resident_v: [B, H_kv, n_resident, 128], attended together with the listed pages."""
        if out is None:
            out = torch.empty((self.batch, self.n_kv_heads * self.group_size, 128), dtype=torch.float32,
                              device=self.device)
        ice_attend_resident(self.handle, q, ids, n_sel, int(ids.shape[-1]), resident_k, resident_v,
                            int(resident_k.shape[-2]), out, stream)
        return out

    def select_attend_resident(self, q, token_budget, resident_k, resident_v, ids=None, n_sel=None, out=None, stream=None):
        if ids is None:
            ids, n_sel = self._sel_buffers(token_budget)
        if out is None:
            out = torch.empty((self.batch, self.n_kv_heads * self.group_size, 128), dtype=torch.float32,
                              device=self.device)
        ice_select_attend_resident(self.handle, q, token_budget, resident_k, resident_v, int(resident_k.shape[-2]), ids,
                                   n_sel, out, stream)
        return ids, n_sel, out

    def selected_tokens(self, ids, n_sel, stream=None):
        """Sequence positions of the tokens of the listed pages: (token_pos [B, H_kv, P * page_size], n_tok)."""
        P = int(ids.shape[-1])
        pos = torch.empty((self.batch, self.n_kv_heads, P * self.page_size), dtype=torch.int32, device=self.device)
        n_tok = torch.empty((self.batch, self.n_kv_heads), dtype=torch.int32, device=self.device)
        ice_selected_tokens(self.handle, ids, n_sel, P, pos, n_tok, stream)
        return pos, n_tok

    def attend_tokens(self, q, K, V, token_pos, n_tok, out=None, stream=None):
        """Attention over rows token_pos[..., :n_tok] of a dense cache K, V [B, H_kv, n_rows, 128]."""
        if out is None:
            out = torch.empty((self.batch, self.n_kv_heads * self.group_size, 128), dtype=torch.float32,
                              device=self.device)
        ice_attend_tokens(self.handle, q, K, V, int(K.shape[-2]), token_pos, n_tok, int(token_pos.shape[-1]), out, stream)
        return out

    def select_hier(self, q, token_budget, n_probe, attend=True, ids=None, n_sel=None, out=None, stream=None, n_refine=0):
        """Staged selection (+ attention in the same launch when attend is true); n_refine > 0 re-ranks
        the n_refine best pages by their best key.
        -> (ids, n_sel, scores, clusters, out or None)."""
        if ids is None:
            ids, n_sel = self._sel_buffers(token_budget)
        P = ids.shape[-1]
        scores = torch.empty((self.batch, self.n_kv_heads, P), dtype=torch.float32, device=self.device)
        clusters = torch.empty((self.batch, self.n_kv_heads, n_probe), dtype=torch.int32, device=self.device)
        if attend and out is None:
            out = torch.empty((self.batch, self.n_kv_heads * self.group_size, 128), dtype=torch.float32,
                              device=self.device)
        ice_select_hier(self.handle, q, token_budget, n_probe, ids, n_sel, scores, clusters, out if attend else None,
                        stream, n_refine)
        return ids, n_sel, scores, clusters, (out if attend else None)

    def build_top_level(self, n_top, iters=3, stream=None):
        """A level of n_top nodes above the clusters (dropped again by the next build_index)."""
        ice_build_top_level(self.handle, n_top, iters, stream)

    def select_hier3(self, q, token_budget, n_probe_top, n_probe, attend=True, stream=None, n_refine=0):
        """Three-level selection (+ attention).  -> (ids, n_sel, scores, clusters, tops, out or None)."""
        ids, n_sel = self._sel_buffers(token_budget)
        P = ids.shape[-1]
        scores = torch.empty((self.batch, self.n_kv_heads, P), dtype=torch.float32, device=self.device)
        clusters = torch.empty((self.batch, self.n_kv_heads, n_probe), dtype=torch.int32, device=self.device)
        tops = torch.empty((self.batch, self.n_kv_heads, n_probe_top), dtype=torch.int32, device=self.device)
        out = torch.empty((self.batch, self.n_kv_heads * self.group_size, 128), dtype=torch.float32,
                          device=self.device) if attend else None
        ice_select_hier3(self.handle, q, token_budget, n_probe_top, n_probe, ids, n_sel, scores, clusters, tops, out, stream,
                         n_refine)
        return ids, n_sel, scores, clusters, tops, out

    def export_top_level(self):
        """The level above the clusters as torch tensors aliasing the workspace."""
        v = ice_export_top_level(self.handle)
        base = self.workspace.data_ptr()

        def view(ptr, dtype, shape):
            nb = int(torch.tensor([], dtype=dtype).element_size())
            n = 1
            for x in shape:
                n *= x
            return self.workspace[ptr - base: ptr - base + n * nb].view(dtype).view(*shape)
        U, T = self.U, v.n_top_max
        return {"n_top": v.n_top,
                "top_centroid": view(v.top_centroid, torch.float32, (U, T, 128))[:, :v.n_top],
                "top_centroid_bf16": view(v.top_centroid_bf16, torch.int16, (U, T, 128)),
                "top_of": view(v.top_of, torch.int32, (U, self.n_clusters)),
                "top_count": view(v.top_count, torch.int32, (U, T))[:, :v.n_top],
                "top_init": view(v.top_init, torch.int32, (U, T))[:, :v.n_top]}

    def export_geometry(self):
        """The extra coordinate of the transformed-key geometry as torch tensors aliasing the workspace
        (None when the index clusters on the raw keys)."""
        v = ice_export_geometry(self.handle)
        if v.geometry == ICE_GEOMETRY_RAW:
            return None
        iv = ice_export_index(self.handle)
        base = self.workspace.data_ptr()

        def view(ptr, dtype, shape):
            nb = int(torch.tensor([], dtype=dtype).element_size())
            n = 1
            for x in shape:
                n *= x
            return self.workspace[ptr - base: ptr - base + n * nb].view(dtype).view(*shape)
        U = self.U
        return {"key_extra": view(v.key_extra, torch.int16, (U, iv.max_tokens)),
                "centroid_extra": view(v.centroid_extra, torch.float32, (U, iv.n_clusters)),
                "cluster_sum_extra": view(v.cluster_sum_extra, torch.float32, (U, iv.n_clusters)),
                "radius_sq": view(v.radius_sq, torch.float32, (U,)),
                "assign_centroid_extra_bf16": view(v.assign_centroid_extra_bf16, torch.int16, (U, iv.cpad))}

    def export(self):
        """dict of torch tensors aliasing the workspace (no copy) plus the view itself under 'view'."""
        v = ice_export_index(self.handle)
        base = self.workspace.data_ptr()
        out = {"view": v}
        for name, (dtype, shape_fn) in _VIEW_FIELDS.items():
            shape = shape_fn(v)
            nbytes = int(torch.tensor([], dtype=dtype).element_size())
            for s in shape:
                nbytes *= s
            off = getattr(v, name) - base
            out[name] = self.workspace[off:off + nbytes].view(dtype).view(shape)
        return out

    def import_arrays(self, arrays: dict, n_tokens: int, stream=None):
        """arrays: name -> device tensor for every field of IMPORT_FIELDS, laid out as in the view."""
        v = IceIndexView()
        v.n_units, v.group_size, v.head_dim = self.U, self.group_size, 128
        v.page_size, v.n_clusters = self.page_size, self.n_clusters
        v.cpad = (self.n_clusters + 31) // 32 * 32
        v.max_pages = self.max_tokens // self.page_size + self.n_clusters
        v.max_tokens, v.n_tokens = self.max_tokens, n_tokens
        for name in IMPORT_FIELDS:
            setattr(v, name, _ptr(arrays[name]))
        ice_import_index(self.handle, v, stream)

    def debug_assign(self, K, centroids_bf16, with_best=True, stream=None):
        n, Cn = K.shape[-2], centroids_bf16.shape[-2]
        a = torch.empty((self.U, n), dtype=torch.int32, device=self.device)
        best = torch.empty((self.U, n), dtype=torch.float32, device=self.device) if with_best else None
        ice_debug_assign(self.handle, K, n, centroids_bf16, Cn, a, best, stream)
        return a, best
