"""ctypes binding of libdg4.so: argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

_P = ctypes.c_void_p
_I64 = ctypes.c_int64
_I32 = ctypes.c_int32

DG4_F32, DG4_BF16 = 0, 1
DG4_NO_EPILOGUE = 1
DG4_PER_LEVEL = 2
DG4_BOUNDED_KV = 4
DG4_FFN = 8
DG4_LEVEL_ORDER = 16
DG4_PROFILE = 32
DG4_TIME_SWEEP = 64
DG4_WEIGHTS_PACKED = 128
ARRAYS = {"level": (0, np.int32), "order": (1, np.int32), "level_ptr": (2, np.int64),
          "nbr_ptr": (3, np.int64), "nbr_idx": (4, np.int32), "nbr_rel": (5, np.uint8),
          "flow_order": (6, np.int32), "flow_tile_ptr": (7, np.int64),
          "out_and": (8, np.int32), "out_not": (9, np.int32),
          "pair_order": (10, np.int32), "pair_tile_ptr": (11, np.int64),
          "cone_root": (12, np.int32), "cone_group_level": (13, np.int32), "cone_group_ptr": (14, np.int64),
          "stage": (15, np.int32), "copy_of": (16, np.int32), "last_copy": (17, np.int32)}
STATUS = {0: "OK", -1: "EINVAL", -2: "ERANGE", -3: "EFANIN", -4: "ECYCLE", -5: "EHINT",
          -6: "EUNSUPPORTED", -7: "ENOMEM", -8: "EWORKSPACE", -9: "EHIP", -10: "EABORTED"}


class DG4Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        self.name = STATUS.get(status, str(status))
        super().__init__(f"{where}: {self.name} ({lib().dg4_strerror(status).decode()})")


class _Cfg(ctypes.Structure):
    _fields_ = [("hidden", _I32), ("heads", _I32), ("hops", _I32), ("n_layers", _I32),
                ("dtype", _I32), ("flags", ctypes.c_uint32), ("ln_eps", ctypes.c_float),
                ("spin_limit", ctypes.c_uint32)]


@dataclass
class LayerConfig:
    hidden: int
    heads: int
    hops: int
    n_layers: int = 1
    dtype: str = "bf16"          # "f32" | "bf16"
    epilogue: bool = True
    ln_eps: float = 1e-5
    per_level: bool = False      # launch level by level instead of the persistent sweep kernel
    bounded_kv: bool = False     # no K|V store: one level's frontier is projected when the level is processed
    ffn: bool = False            # every layer ends with the feed-forward sub-block (weights W1, W2 per layer)
    level_order: bool = False    # whole-graph sweeps follow the graph's own levels, not the dependency-driven order
    profile: bool = False        # phase timers of the specialised persistent kernel (dg4_layer_profile)
    time_sweep: bool = False     # events around the persistent kernel (dg4_sweep_elapsed_ms)
    weights_packed: bool = False # reuse the packed weights the previous call left in the workspace
    spin_limit: int = 0          # polls before a persistent sweep gives up on a dependency (0: default)

    def c(self) -> _Cfg:
        return _Cfg(self.hidden, self.heads, self.hops, self.n_layers,
                    DG4_F32 if self.dtype == "f32" else DG4_BF16,
                    (0 if self.epilogue else DG4_NO_EPILOGUE) | (DG4_PER_LEVEL if self.per_level else 0) |
                    (DG4_BOUNDED_KV if self.bounded_kv else 0) | (DG4_FFN if self.ffn else 0) |
                    (DG4_LEVEL_ORDER if self.level_order else 0) | (DG4_PROFILE if self.profile else 0) |
                    (DG4_TIME_SWEEP if self.time_sweep else 0) | (DG4_WEIGHTS_PACKED if self.weights_packed else 0),
                    self.ln_eps, self.spin_limit)


_lib = None


def library_path() -> str:
    return _build.LIB


def lib():
    """The loaded C library. Built first if absent; a failure to load is fatal by design."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build()
        L = ctypes.CDLL(_build.LIB)
        L.dg4_strerror.restype = ctypes.c_char_p
        L.dg4_strerror.argtypes = [ctypes.c_int]
        L.dg4_build_levels.restype = ctypes.c_int
        L.dg4_build_levels.argtypes = [_I64, _I64, _P, _P, _P, _I32, _P, ctypes.POINTER(_P)]
        L.dg4_graph_array.restype = ctypes.c_int
        L.dg4_build_partitioned.restype = ctypes.c_int
        L.dg4_build_partitioned.argtypes = [_I64, _I64, _P, _P, _P, _I32, _P, _I32, _I32, _I32, ctypes.POINTER(_P)]
        L.dg4_build_levels_device.restype = ctypes.c_int
        L.dg4_build_levels_device.argtypes = [_I64, _I64, _P, _P, _P, _I32, _P, _P, ctypes.POINTER(_P)]
        L.dg4_build_partitioned_device.restype = ctypes.c_int
        L.dg4_build_partitioned_device.argtypes = [_I64, _I64, _P, _P, _P, _I32, _P, _I32, _I32, _P, ctypes.POINTER(_P)]
        L.dg4_graph_array.argtypes = [_P, ctypes.c_int, ctypes.POINTER(_P), ctypes.POINTER(_I64)]
        L.dg4_graph_info.restype = ctypes.c_int
        L.dg4_graph_info.argtypes = [_P, ctypes.POINTER(_I64), ctypes.POINTER(_I64), ctypes.POINTER(_I64),
                                     ctypes.POINTER(_I32)]
        L.dg4_graph_upload.restype = ctypes.c_int
        L.dg4_graph_upload.argtypes = [_P]
        L.dg4_graph_free.restype = None
        L.dg4_graph_free.argtypes = [_P]
        L.dg4_proj_workspace_bytes.restype = _I64
        L.dg4_proj_workspace_bytes.argtypes = [ctypes.POINTER(_Cfg)]
        L.dg4_layer_workspace_bytes.restype = _I64
        L.dg4_ffn_workspace_bytes.restype = _I64
        L.dg4_ffn_workspace_bytes.argtypes = [ctypes.POINTER(_Cfg)]
        L.dg4_ffn_fwd.restype = ctypes.c_int
        L.dg4_ffn_fwd.argtypes = [ctypes.POINTER(_Cfg), _P, _I64, _I64, _P, _P, _P, _P, _I64, _P]
        L.dg4_layer_workspace_bytes.argtypes = [ctypes.POINTER(_Cfg), _P]
        L.dg4_qkv_proj.restype = ctypes.c_int
        L.dg4_qkv_proj.argtypes = [ctypes.POINTER(_Cfg), _P, _I64, _I64, _P, _P, _P, _P, _P, _I64, _P]
        L.dg4_qkv_proj_static.restype = ctypes.c_int
        L.dg4_qkv_proj_static.argtypes = [ctypes.POINTER(_Cfg), _P, _I64, _I64, _P, _P, _P, _P, _P]
        L.dg4_static_scratch_bytes.restype = _I64
        L.dg4_static_scratch_bytes.argtypes = []
        L.dg4_struct_encode.restype = ctypes.c_int
        L.dg4_struct_encode.argtypes = [ctypes.POINTER(_Cfg), _P, _P, _P, _P, _P]
        L.dg4_sparse_attn_fwd.restype = ctypes.c_int
        L.dg4_sparse_attn_fwd.argtypes = [ctypes.POINTER(_Cfg), _P, _I64, _I64, _P, _P, _P, _P, _P, _P]
        L.dg4_layer_fwd.restype = ctypes.c_int
        L.dg4_layer_fwd.argtypes = [ctypes.POINTER(_Cfg), _P, _P, ctypes.POINTER(_P), _I32, _I32, _P, _P, _I64, _P]
        L.dg4_sweep_elapsed_ms.restype = ctypes.c_int
        L.dg4_sweep_elapsed_ms.argtypes = [ctypes.POINTER(ctypes.c_float)]
        L.dg4_layer_status.restype = ctypes.c_int
        L.dg4_layer_status.argtypes = [ctypes.POINTER(_Cfg), _P, _P]
        L.dg4_layer_profile.restype = ctypes.c_int
        L.dg4_layer_profile.argtypes = [ctypes.POINTER(_Cfg), _P, _P, ctypes.POINTER(ctypes.c_uint64),
                                        ctypes.POINTER(ctypes.c_uint32)]
        _lib = L
    return _lib


def _check(rc: int, where: str):
    if rc != 0:
        raise DG4Error(int(rc), where)


class Graph:
    """Owner of a dg4_graph handle; tables are exposed as numpy copies."""

    def __init__(self, handle: int):
        self._h = _P(handle)
        n, nl, nnz, hops = _I64(), _I64(), _I64(), _I32()
        _check(lib().dg4_graph_info(self._h, n, nl, nnz, hops), "dg4_graph_info")
        self.n, self.n_levels, self.nnz, self.hops = n.value, nl.value, nnz.value, hops.value

    @property
    def handle(self):
        return self._h

    def array(self, name: str) -> np.ndarray:
        which, dtype = ARRAYS[name]
        ptr, cnt = _P(), _I64()
        _check(lib().dg4_graph_array(self._h, which, ptr, cnt), "dg4_graph_array")
        if cnt.value == 0:
            return np.empty(0, dtype=dtype)
        buf = (ctypes.c_char * (cnt.value * np.dtype(dtype).itemsize)).from_address(ptr.value)
        return np.frombuffer(buf, dtype=dtype).copy()

    def upload(self):
        _check(lib().dg4_graph_upload(self._h), "dg4_graph_upload")

    def close(self):
        if self._h:
            lib().dg4_graph_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def dg4_build_levels(n_nodes, edge_src, edge_dst, edge_inv, hops, level_hint=None) -> Graph:
    src = np.ascontiguousarray(edge_src, dtype=np.int32)
    dst = np.ascontiguousarray(edge_dst, dtype=np.int32)
    inv = np.ascontiguousarray(edge_inv, dtype=np.uint8)
    if not (len(src) == len(dst) == len(inv)):
        raise DG4Error(-1, "dg4_build_levels")
    hint = None if level_hint is None else np.ascontiguousarray(level_hint, dtype=np.int32)
    if hint is not None and len(hint) != n_nodes:
        raise DG4Error(-1, "dg4_build_levels")
    out = _P()
    rc = lib().dg4_build_levels(n_nodes, len(src), src.ctypes.data, dst.ctypes.data, inv.ctypes.data, hops,
                                hint.ctypes.data if hint is not None else None, ctypes.byref(out))
    _check(rc, "dg4_build_levels")
    return Graph(out.value)


def dg4_build_partitioned(n_nodes, edge_src, edge_dst, edge_inv, hops, stride, batch_cones, level_hint=None,
                          marks=True) -> Graph:
    src = np.ascontiguousarray(edge_src, dtype=np.int32)
    dst = np.ascontiguousarray(edge_dst, dtype=np.int32)
    inv = np.ascontiguousarray(edge_inv, dtype=np.uint8)
    if not (len(src) == len(dst) == len(inv)):
        raise DG4Error(-1, "dg4_build_partitioned")
    hint = None if level_hint is None else np.ascontiguousarray(level_hint, dtype=np.int32)
    if hint is not None and len(hint) != n_nodes:
        raise DG4Error(-1, "dg4_build_partitioned")
    out = _P()
    rc = lib().dg4_build_partitioned(n_nodes, len(src), src.ctypes.data, dst.ctypes.data, inv.ctypes.data, hops,
                                     hint.ctypes.data if hint is not None else None, stride, batch_cones,
                                     int(marks), ctypes.byref(out))
    _check(rc, "dg4_build_partitioned")
    return Graph(out.value)


def dg4_build_levels_device(n_nodes, edge_src, edge_dst, edge_inv, hops, level_hint=None) -> Graph:
    """dg4_build_levels on the GPU: edge_src/edge_dst (int32), edge_inv (uint8) and level_hint (int32 or
    None) are device tensors."""
    import torch
    assert edge_src.dtype == torch.int32 and edge_dst.dtype == torch.int32 and edge_inv.dtype == torch.uint8
    assert edge_src.is_cuda and edge_dst.is_cuda and edge_inv.is_cuda
    assert edge_src.is_contiguous() and edge_dst.is_contiguous() and edge_inv.is_contiguous()
    if not (edge_src.numel() == edge_dst.numel() == edge_inv.numel()):
        raise DG4Error(-1, "dg4_build_levels_device")
    if level_hint is not None:
        assert level_hint.dtype == torch.int32 and level_hint.is_cuda and level_hint.is_contiguous()
        if level_hint.numel() != n_nodes:
            raise DG4Error(-1, "dg4_build_levels_device")
    out = _P()
    rc = lib().dg4_build_levels_device(n_nodes, edge_src.numel(), edge_src.data_ptr(), edge_dst.data_ptr(),
                                       edge_inv.data_ptr(), hops,
                                       level_hint.data_ptr() if level_hint is not None else None,
                                       _stream(), ctypes.byref(out))
    _check(rc, "dg4_build_levels_device")
    return Graph(out.value)


def dg4_build_partitioned_device(n_nodes, edge_src, edge_dst, edge_inv, hops, stride, batch_cones, level_hint=None) -> Graph:
    """dg4_build_partitioned (with marks) on the GPU: the edge list and the hint are device tensors."""
    import torch
    assert edge_src.dtype == torch.int32 and edge_dst.dtype == torch.int32 and edge_inv.dtype == torch.uint8
    assert edge_src.is_cuda and edge_dst.is_cuda and edge_inv.is_cuda
    assert edge_src.is_contiguous() and edge_dst.is_contiguous() and edge_inv.is_contiguous()
    if not (edge_src.numel() == edge_dst.numel() == edge_inv.numel()):
        raise DG4Error(-1, "dg4_build_partitioned_device")
    if level_hint is not None:
        assert level_hint.dtype == torch.int32 and level_hint.is_cuda and level_hint.is_contiguous()
        if level_hint.numel() != n_nodes:
            raise DG4Error(-1, "dg4_build_partitioned_device")
    out = _P()
    rc = lib().dg4_build_partitioned_device(n_nodes, edge_src.numel(), edge_src.data_ptr(), edge_dst.data_ptr(),
                                            edge_inv.data_ptr(), hops,
                                            level_hint.data_ptr() if level_hint is not None else None,
                                            stride, batch_cones, _stream(), ctypes.byref(out))
    _check(rc, "dg4_build_partitioned_device")
    return Graph(out.value)


def dg4_proj_workspace_bytes(cfg: LayerConfig) -> int:
    c = cfg.c()
    r = lib().dg4_proj_workspace_bytes(ctypes.byref(c))
    if r < 0:
        raise DG4Error(int(r), "dg4_proj_workspace_bytes")
    return int(r)


def dg4_ffn_workspace_bytes(cfg: LayerConfig) -> int:
    c = cfg.c()
    r = lib().dg4_ffn_workspace_bytes(ctypes.byref(c))
    if r < 0:
        raise DG4Error(int(r), "dg4_ffn_workspace_bytes")
    return int(r)


def dg4_layer_workspace_bytes(cfg: LayerConfig, g: Graph) -> int:
    c = cfg.c()
    r = lib().dg4_layer_workspace_bytes(ctypes.byref(c), g.handle)
    if r < 0:
        raise DG4Error(int(r), "dg4_layer_workspace_bytes")
    return int(r)


def _stream():
    import torch
    return _P(torch.cuda.current_stream().cuda_stream)


def _ws(nbytes: int, like):
    import torch
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=like.device)


def dg4_qkv_proj(cfg: LayerConfig, S, Wqkv, Q, K, V, row_begin=0, row_end=None, workspace=None):
    """Q, K, V rows [row_begin,row_end) = S rows x [Wq | Wk | Wv] (device tensors, in place)."""
    row_end = S.shape[0] if row_end is None else row_end
    ws = _ws(dg4_proj_workspace_bytes(cfg), S) if workspace is None else workspace
    c = cfg.c()
    rc = lib().dg4_qkv_proj(ctypes.byref(c), S.data_ptr(), row_begin, row_end, Wqkv.data_ptr(),
                            Q.data_ptr(), K.data_ptr(), V.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "dg4_qkv_proj")


def dg4_static_scratch_bytes() -> int:
    return int(lib().dg4_static_scratch_bytes())


def dg4_qkv_proj_static(cfg: LayerConfig, S, Wqkv, Q, K, V, row_begin=0, row_end=None):
    """dg4_qkv_proj without a workspace: the library's own device array takes the packed weight."""
    row_end = S.shape[0] if row_end is None else row_end
    c = cfg.c()
    rc = lib().dg4_qkv_proj_static(ctypes.byref(c), S.data_ptr(), row_begin, row_end, Wqkv.data_ptr(),
                                   Q.data_ptr(), K.data_ptr(), V.data_ptr(), _stream())
    _check(rc, "dg4_qkv_proj_static")


def dg4_ffn_fwd(cfg: LayerConfig, S, W1, W2, Out, row_begin=0, row_end=None, workspace=None):
    """Out rows [row_begin,row_end) = LayerNorm(S + relu(S W1) W2) (device tensors, Out in place)."""
    row_end = S.shape[0] if row_end is None else row_end
    ws = _ws(dg4_ffn_workspace_bytes(cfg), S) if workspace is None else workspace
    c = cfg.c()
    rc = lib().dg4_ffn_fwd(ctypes.byref(c), S.data_ptr(), row_begin, row_end, W1.data_ptr(), W2.data_ptr(),
                           Out.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "dg4_ffn_fwd")


def dg4_struct_encode(cfg: LayerConfig, g: Graph, X, emb, Xout):
    """Xout = X + structural encoding (level, OutAND, OutNOT through three linear layers); emb float [6, hidden]."""
    c = cfg.c()
    rc = lib().dg4_struct_encode(ctypes.byref(c), g.handle, X.data_ptr(), emb.data_ptr(), Xout.data_ptr(), _stream())
    _check(rc, "dg4_struct_encode")


def dg4_sparse_attn_fwd(cfg: LayerConfig, g: Graph, Q, K, V, rel_bias, A, row_begin=0, row_end=None):
    row_end = g.n if row_end is None else row_end
    c = cfg.c()
    rc = lib().dg4_sparse_attn_fwd(ctypes.byref(c), g.handle, row_begin, row_end, Q.data_ptr(), K.data_ptr(),
                                   V.data_ptr(), rel_bias.data_ptr(), A.data_ptr(), _stream())
    _check(rc, "dg4_sparse_attn_fwd")


def dg4_layer_fwd(cfg: LayerConfig, g: Graph, X, weights, Hout, level_begin=0, level_end=None, workspace=None):
    """weights: per layer (Wqkv, Wo, rel_bias) device tensors, or (Wqkv, Wo, rel_bias, W1, W2) with
    cfg.ffn. Hout is written in place."""
    assert all(len(layer) == (5 if cfg.ffn else 3) for layer in weights) and len(weights) == cfg.n_layers
    level_end = g.n_levels if level_end is None else level_end
    ws = _ws(dg4_layer_workspace_bytes(cfg, g), X) if workspace is None else workspace
    flat = [t.data_ptr() for layer in weights for t in layer]
    arr = (_P * len(flat))(*flat)
    c = cfg.c()
    rc = lib().dg4_layer_fwd(ctypes.byref(c), g.handle, X.data_ptr(), arr, level_begin, level_end,
                             Hout.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "dg4_layer_fwd")
    return ws


def dg4_layer_status(cfg: LayerConfig, g: Graph, workspace, check=True) -> int:
    """Status of the last dg4_layer_fwd on `workspace` (synchronise first): 0, or raises / returns EABORTED."""
    c = cfg.c()
    rc = int(lib().dg4_layer_status(ctypes.byref(c), g.handle, workspace.data_ptr()))
    if check:
        _check(rc, "dg4_layer_status")
    return rc


def dg4_layer_profile(cfg: LayerConfig, g: Graph, workspace):
    """(aborted, ticks[8]) left in `workspace` by the last persistent sweep (synchronise first)."""
    ticks = (ctypes.c_uint64 * 8)()
    aborted = ctypes.c_uint32()
    c = cfg.c()
    _check(lib().dg4_layer_profile(ctypes.byref(c), g.handle, workspace.data_ptr(), ticks, ctypes.byref(aborted)),
           "dg4_layer_profile")
    return int(aborted.value), [int(t) for t in ticks]


def dg4_sweep_elapsed_ms() -> float:
    """Device time of the last persistent sweep kernel launched with cfg.time_sweep."""
    ms = ctypes.c_float()
    _check(lib().dg4_sweep_elapsed_ms(ctypes.byref(ms)), "dg4_sweep_elapsed_ms")
    return float(ms.value)
