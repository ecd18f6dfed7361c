"""Helpers shared by the GPU parity tests: upload/download and mirroring an exported GPU index into
an OracleIndex (plain array copies; no arithmetic of the method lives here)."""
import numpy as np
import torch

from oracle import ice_oracle as orc

D = 128
STATE_FIELDS = ("n_pages", "Kp", "Vp", "page_cluster", "page_fill", "page_pos", "cluster_tail", "cluster_cnt",
                "cluster_sum", "centroid", "page_sum", "rep")


def up(a: np.ndarray, dev="cuda:0") -> torch.Tensor:
    """numpy -> device tensor; uint16 bf16 bit patterns travel as int16."""
    a = np.ascontiguousarray(a)
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)


def down(t: torch.Tensor) -> np.ndarray:
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


def export_np(ix) -> dict:
    torch.cuda.synchronize()
    ex = ix.export()
    out = {k: down(v).copy() for k, v in ex.items() if k != "view"}
    out["n_tokens"] = ex["view"].n_tokens
    return out


def oracle_from_export(ix, ex: dict) -> orc.OracleIndex:
    """An OracleIndex holding exactly the bits the GPU index holds."""
    o = orc.OracleIndex(ix.U, ix.group_size, ix.page_size, ix.n_clusters, ix.max_tokens)
    for name in STATE_FIELDS:
        getattr(o, name)[...] = ex[name]
    o.n_tokens[:] = ex["n_tokens"]
    return o


def oracle_arrays_to_device(o: orc.OracleIndex, dev="cuda:0") -> dict:
    return {name: up(getattr(o, name), dev) for name in STATE_FIELDS}


def valid_slot_mask(fill: np.ndarray, s: int) -> np.ndarray:
    return np.arange(s)[None, :] < fill[:, None]
