"""ctypes front end of the CPU oracle (oracle/dg4_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg. The GPU package never imports this module.
All arithmetic is in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libdg4oracle.so")
_SRC = os.path.join(_HERE, "dg4_oracle.c")

STORE = {"f64": 0, "f32": 1, "bf16": 2}
ERRORS = {-1: "EINVAL", -2: "ERANGE", -3: "EFANIN", -4: "ECYCLE", -5: "EHINT", -6: "ENOMEM"}


class OracleError(ValueError):
    def __init__(self, code: int):
        super().__init__(ERRORS.get(code, str(code)))
        self.code = code
        self.name = ERRORS.get(code, str(code))


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math: arithmetic stays in the written order)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"])
    return _SO


_lib = None
_P = ctypes.c_void_p
_I64 = ctypes.c_int64
_I32 = ctypes.c_int32
_F64 = ctypes.c_double


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.orc_validate.restype = ctypes.c_int
        lib.orc_validate.argtypes = [_I64, _I64, _P, _P, _P]
        lib.orc_levels.restype = ctypes.c_int
        lib.orc_levels.argtypes = [_I64, _I64, _P, _P, _P]
        lib.orc_check_hint.restype = ctypes.c_int
        lib.orc_check_hint.argtypes = [_I64, _I64, _P, _P, _P]
        lib.orc_order.restype = None
        lib.orc_order.argtypes = [_I64, _P, _I32, _P, _P]
        lib.orc_cone_csr.restype = _I64
        lib.orc_cone_csr.argtypes = [_I64, _I64, _P, _P, _P, _I32, _P, _P, _P]
        lib.orc_qkv_proj.restype = None
        lib.orc_qkv_proj.argtypes = [_I64, _I32, _P, _P, _P, _P, _P]
        lib.orc_sparse_attn.restype = None
        lib.orc_sparse_attn.argtypes = [_I64, _I32, _I32, _I64, _I64, _P, _P, _P, _P, _P, _P, _P, _P, _P]
        lib.orc_layer_fwd.restype = ctypes.c_int
        lib.orc_layer_fwd.argtypes = [_I64, _I32, _I32, _I32, _I32, _I32, _F64, _I32,
                                      _P, _P, _P, _P, _P, _P, _P, _P, _I32, _I32, _P, _P, _P, _P]
        lib.orc_layer_nodes.restype = ctypes.c_int
        lib.orc_layer_nodes.argtypes = [_I64, _I32, _I32, _I32, _I32, _I32, _F64,
                                        _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _I64, _P]
        lib.orc_ffn.restype = ctypes.c_int
        lib.orc_ffn.argtypes = [_I64, _I32, _P, _P, _P, _F64, _I32, _P]
        lib.orc_out_degrees.restype = None
        lib.orc_out_degrees.argtypes = [_I64, _I64, _P, _P, _P, _P, _P]
        lib.orc_struct_encode.restype = None
        lib.orc_struct_encode.argtypes = [_I64, _I32, _P, _P, _P, _P, _P, _I32, _P]
        lib.orc_threads.restype = ctypes.c_int
        lib.orc_threads.argtypes = []
        lib.orc_partition.restype = ctypes.c_void_p
        lib.orc_partition.argtypes = [_I64, _I64, _P, _P, _I32, _I32, _P, _P]
        lib.orc_cones_sizes.restype = None
        lib.orc_cones_sizes.argtypes = [_P, _P, _P, _P]
        lib.orc_cones_copy.restype = None
        lib.orc_cones_copy.argtypes = [_P, _P, _P, _P, _P, _P]
        lib.orc_cones_free.restype = None
        lib.orc_cones_free.argtypes = [_P]
        lib.orc_partitioned_fwd.restype = ctypes.c_int
        lib.orc_partitioned_fwd.argtypes = [_I64, _I32, _I32, _I32, _I32, _I32, _F64,
                                            _P, _P, _P, _P, _P, _P,
                                            _P, _P, _P, _P,
                                            _I64, _P, _P, _P, _I32, _I32, _I32,
                                            _P, _P, _P, _P]
        _lib = lib
    return _lib


def threads() -> int:
    """Threads the oracle's per-level loops use (OpenMP)."""
    return int(_load().orc_threads())


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a):
    return a.ctypes.data if a is not None else None


@dataclass
class Graph:
    n: int
    level: np.ndarray        # int32 [N]  Eq. 1 level, or the validated hint
    order: np.ndarray        # int32 [N]  ids by (level, id)
    level_ptr: np.ndarray    # int64 [max_level + 2]
    nbr_ptr: np.ndarray      # int64 [N + 1]
    nbr_idx: np.ndarray      # int32 [NNZ] ascending id inside a row
    nbr_rel: np.ndarray      # uint8 [NNZ] 0 self, 1 fanin, 2 inverted fanin, 3 virtual
    hops: int = -1           # cone depth k the rows were built with

    @property
    def n_levels(self) -> int:
        return len(self.level_ptr) - 1


def levels(n, src, dst) -> np.ndarray:
    """Eq. 1 logic levels."""
    src, dst = _c(src, np.int32), _c(dst, np.int32)
    lev = np.empty(n, dtype=np.int32)
    rc = _load().orc_levels(n, len(src), _ptr(src), _ptr(dst), _ptr(lev))
    if rc:
        raise OracleError(rc)
    return lev


def build_levels(n, src, dst, inv, hops, level_hint=None) -> Graph:
    """Validation, levels (Eq. 1 or checked hint), (level,id) order, cone CSR."""
    lib = _load()
    src, dst, inv = _c(src, np.int32), _c(dst, np.int32), _c(inv, np.uint8)
    e = len(src)
    if len(dst) != e or len(inv) != e:
        raise OracleError(-1)
    rc = lib.orc_validate(n, e, _ptr(src), _ptr(dst), _ptr(inv))
    if rc:
        raise OracleError(rc)
    lev = levels(n, src, dst)           # also detects cycles
    if level_hint is not None:
        hint = _c(level_hint, np.int32)
        if len(hint) != n:
            raise OracleError(-1)
        rc = lib.orc_check_hint(n, e, _ptr(src), _ptr(dst), _ptr(hint))
        if rc:
            raise OracleError(rc)
        lev = hint.copy()
    max_level = int(lev.max()) if n else 0
    order = np.empty(n, dtype=np.int32)
    level_ptr = np.empty(max_level + 2, dtype=np.int64)
    lib.orc_order(n, _ptr(lev), max_level, _ptr(order), _ptr(level_ptr))
    nbr_ptr = np.empty(n + 1, dtype=np.int64)
    nnz = lib.orc_cone_csr(n, e, _ptr(src), _ptr(dst), _ptr(inv), hops, _ptr(nbr_ptr), None, None)
    if nnz < 0:
        raise OracleError(int(nnz))
    nbr_idx = np.empty(nnz, dtype=np.int32)
    nbr_rel = np.empty(nnz, dtype=np.uint8)
    lib.orc_cone_csr(n, e, _ptr(src), _ptr(dst), _ptr(inv), hops, _ptr(nbr_ptr), _ptr(nbr_idx), _ptr(nbr_rel))
    return Graph(n, lev, order, level_ptr, nbr_ptr, nbr_idx, nbr_rel, int(hops))


def qkv_proj(S, W):
    """Q, K, V = S @ W[:, :d], S @ W[:, d:2d], S @ W[:, 2d:] in double."""
    S, W = _c(S, np.float32), _c(W, np.float32)
    rows, d = S.shape
    assert W.shape == (d, 3 * d) and d <= 1024
    Q, K, V = (np.empty((rows, d), dtype=np.float64) for _ in range(3))
    _load().orc_qkv_proj(rows, d, _ptr(S), _ptr(W), _ptr(Q), _ptr(K), _ptr(V))
    return Q, K, V


def sparse_attn(g: Graph, heads, Q, K, V, rel_bias, row_begin=0, row_end=None, want_alpha=False):
    """Scores, segmented softmax, aggregation on given Q, K, V (rows = node ids)."""
    Q, K, V = _c(Q, np.float32), _c(K, np.float32), _c(V, np.float32)
    rel_bias = _c(rel_bias, np.float32)
    n, d = Q.shape
    row_end = n if row_end is None else row_end
    A = np.zeros((n, d), dtype=np.float64)
    alpha = np.zeros((len(g.nbr_idx), heads), dtype=np.float64) if want_alpha else None
    _load().orc_sparse_attn(n, d, heads, row_begin, row_end, _ptr(Q), _ptr(K), _ptr(V), _ptr(rel_bias),
                            _ptr(g.nbr_ptr), _ptr(g.nbr_idx), _ptr(g.nbr_rel), _ptr(A), _ptr(alpha))
    return (A, alpha) if want_alpha else A


def _stack(ws, shape):
    a = np.ascontiguousarray(np.stack([np.asarray(w, dtype=np.float32) for w in ws]))
    assert a.shape[1:] == shape, (a.shape, shape)
    return a


def _ffn(w1, w2, nl, d):
    if w1 is None and w2 is None:
        return None, None
    assert w1 is not None and w2 is not None and len(w1) == nl and len(w2) == nl
    return _stack(w1, (d, 4 * d)), _stack(w2, (4 * d, d))


def layer_fwd(g: Graph, x, wqkv, wo, rel_bias, heads, *, store="f64", epilogue=True, ln_eps=1e-5,
              memo=True, level_begin=0, level_end=None, H_init=None, w1=None, w2=None):
    """The full level sweep. wqkv / wo / rel_bias (and w1 / w2 of the feed-forward sub-block,
    if any) are per-layer lists. Returns H [N,d] float64."""
    x = _c(x, np.float32)
    n, d = x.shape
    nl = len(wqkv)
    Wqkv, Wo, B = _stack(wqkv, (d, 3 * d)), _stack(wo, (d, d)), _stack(rel_bias, (heads, 4))
    W1, W2 = _ffn(w1, w2, nl, d)
    level_end = g.n_levels if level_end is None else level_end
    H = np.zeros((n, d), dtype=np.float64) if H_init is None else np.array(H_init, dtype=np.float64, order="C")
    rc = _load().orc_layer_fwd(n, d, heads, nl, STORE[store], int(epilogue), float(ln_eps), int(memo),
                               _ptr(x), _ptr(Wqkv), _ptr(Wo), _ptr(B), _ptr(W1), _ptr(W2), _ptr(g.order), _ptr(g.level_ptr),
                               level_begin, level_end, _ptr(g.nbr_ptr), _ptr(g.nbr_idx), _ptr(g.nbr_rel), _ptr(H))
    if rc:
        raise OracleError(rc)
    return H


def layer_nodes(g: Graph, x, wqkv, wo, rel_bias, heads, Hsrc, nodes, *, store="f64", epilogue=True,
                ln_eps=1e-5, w1=None, w2=None):
    """One step for the listed nodes, sources' final embeddings given in Hsrc [N,d] float32."""
    x, Hsrc = _c(x, np.float32), _c(Hsrc, np.float32)
    n, d = x.shape
    nl = len(wqkv)
    Wqkv, Wo, B = _stack(wqkv, (d, 3 * d)), _stack(wo, (d, d)), _stack(rel_bias, (heads, 4))
    W1, W2 = _ffn(w1, w2, nl, d)
    nodes = _c(nodes, np.int64)
    out = np.empty((len(nodes), d), dtype=np.float64)
    rc = _load().orc_layer_nodes(n, d, heads, nl, STORE[store], int(epilogue), float(ln_eps),
                                 _ptr(x), _ptr(Wqkv), _ptr(Wo), _ptr(B), _ptr(W1), _ptr(W2),
                                 _ptr(g.nbr_ptr), _ptr(g.nbr_idx), _ptr(g.nbr_rel),
                                 _ptr(Hsrc), _ptr(nodes), len(nodes), _ptr(out))
    if rc:
        raise OracleError(rc)
    return out


def ffn(S, w1, w2, *, ln_eps=1e-5, store="f64"):
    """LayerNorm(S + relu(S W1) W2) row by row (reading R16). Returns float64 [rows, d]."""
    S, w1, w2 = _c(S, np.float32), _c(w1, np.float32), _c(w2, np.float32)
    rows, d = S.shape
    assert w1.shape == (d, 4 * d) and w2.shape == (4 * d, d)
    out = np.empty((rows, d), dtype=np.float64)
    rc = _load().orc_ffn(rows, d, _ptr(S), _ptr(w1), _ptr(w2), float(ln_eps), STORE[store], _ptr(out))
    if rc:
        raise OracleError(rc)
    return out


def out_degrees(n, src, dst, inv):
    """OutAND(v), OutNOT(v) of Eq. 2: AND / NOT gates among the direct fanouts (reading R15)."""
    src, dst, inv = _c(src, np.int32), _c(dst, np.int32), _c(inv, np.uint8)
    out_and, out_not = np.empty(n, dtype=np.int32), np.empty(n, dtype=np.int32)
    _load().orc_out_degrees(n, len(src), _ptr(src), _ptr(dst), _ptr(inv), _ptr(out_and), _ptr(out_not))
    return out_and, out_not


def struct_encode(x, level, out_and, out_not, emb, store="f64"):
    """x + SE (Eq. 2); emb [6, d] = w_l, b_l, w_and, b_and, w_not, b_not. Returns float64 [N, d]."""
    x, emb = _c(x, np.float32), _c(emb, np.float32)
    n, d = x.shape
    assert emb.shape == (6, d)
    level, out_and, out_not = _c(level, np.int32), _c(out_and, np.int32), _c(out_not, np.int32)
    out = np.empty((n, d), dtype=np.float64)
    _load().orc_struct_encode(n, d, _ptr(x), _ptr(level), _ptr(out_and), _ptr(out_not), _ptr(emb), STORE[store], _ptr(out))
    return out


@dataclass
class Cones:
    """Algorithm 1's result: the lists cones^l by ascending l, each a run of cones."""
    group_level: np.ndarray   # int32 [G]      level l of each list
    group_ptr: np.ndarray     # int64 [G + 1]  first cone of each list
    cone_root: np.ndarray     # int32 [C]
    cone_ptr: np.ndarray      # int64 [C + 1]  into cone_node
    cone_node: np.ndarray     # int32          gates of each cone, ascending id

    def cone(self, c):
        return self.cone_node[self.cone_ptr[c]:self.cone_ptr[c + 1]]


def partition(g: Graph, src, delta) -> Cones:
    """Algorithm 1 (reading R17) with k = the hops the graph's cone rows were built with."""
    lib = _load()
    src = _c(src, np.int32)
    k = _hops_of(g)
    h = lib.orc_partition(g.n, len(src), _ptr(src), _ptr(g.level), k, int(delta), _ptr(g.nbr_ptr), _ptr(g.nbr_idx))
    if not h:
        raise OracleError(-1)
    try:
        sizes = [ctypes.c_int64() for _ in range(3)]
        lib.orc_cones_sizes(h, *[ctypes.addressof(t) for t in sizes])
        G, C, E = (int(t.value) for t in sizes)
        out = Cones(np.empty(G, np.int32), np.empty(G + 1, np.int64), np.empty(C, np.int32),
                    np.empty(C + 1, np.int64), np.empty(E, np.int32))
        lib.orc_cones_copy(h, _ptr(out.group_level), _ptr(out.group_ptr), _ptr(out.cone_root),
                           _ptr(out.cone_ptr), _ptr(out.cone_node))
    finally:
        lib.orc_cones_free(h)
    return out


def _hops_of(g: Graph) -> int:
    if g.hops < 1:
        raise ValueError("the graph does not say which cone depth its rows were built with")
    return int(g.hops)


def partitioned_fwd(g: Graph, cones: Cones, batch, x, wqkv, wo, rel_bias, heads, *, mark=True, store="f64",
                    epilogue=True, ln_eps=1e-5, w1=None, w2=None, memo=True):
    """Algorithm 2 at inference over Algorithm 1's lists (reading R17).

    Returns (H [N,d] float64, rows, stage_of, n_computed): rows = (ptr, idx, rel) of the
    neighbourhood each gate was (last) computed with, stage_of the running number of the
    mini-batch that did it, n_computed the number of gate computations."""
    x = _c(x, np.float32)
    n, d = x.shape
    nl = len(wqkv)
    Wqkv, Wo, B = _stack(wqkv, (d, 3 * d)), _stack(wo, (d, d)), _stack(rel_bias, (heads, 4))
    W1, W2 = _ffn(w1, w2, nl, d)
    H = np.full((n, d), np.nan, dtype=np.float64)
    kept = np.zeros(len(g.nbr_idx), dtype=np.uint8)
    stage_of = np.full(n, -1, dtype=np.int32)
    n_computed = ctypes.c_int64()
    rc = _load().orc_partitioned_fwd(n, d, heads, nl, STORE[store], int(epilogue), float(ln_eps),
                                     _ptr(x), _ptr(Wqkv), _ptr(Wo), _ptr(B), _ptr(W1), _ptr(W2),
                                     _ptr(g.level), _ptr(g.nbr_ptr), _ptr(g.nbr_idx), _ptr(g.nbr_rel),
                                     len(cones.group_level), _ptr(cones.group_ptr), _ptr(cones.cone_ptr),
                                     _ptr(cones.cone_node), int(batch), int(mark), int(memo),
                                     _ptr(H), _ptr(kept), _ptr(stage_of), ctypes.addressof(n_computed))
    if rc:
        raise OracleError(rc)
    sel = kept.astype(bool)
    cnt = np.add.reduceat(kept.astype(np.int64), g.nbr_ptr[:-1]) if n else np.zeros(0, np.int64)
    ptr = np.concatenate([[0], np.cumsum(cnt)]).astype(np.int64)
    return H, (ptr, g.nbr_idx[sel], g.nbr_rel[sel]), stage_of, int(n_computed.value)
