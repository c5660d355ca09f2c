"""Seeded synthetic workloads (inputs only; none of the method's arithmetic).

Five configurations of And-Inverter Graphs plus Gaussian features and weights.
They stand in for the circuit datasets of the paper (Section "Dataset
Statistic": ITC99, EPFL, OpenABC-D; Section 4.4 scaling circuits), which are
not available offline. Both the CPU oracle's tests and the GPU tests/bench draw
their inputs here, so the two sides see identical bytes.

All floating-point values are returned as float32 numpy arrays; for bf16
configurations every value is already rounded to a bf16-representable number.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libdg4synth.so")
_SRC = os.path.join(_HERE, "synth.c")

BASE_SEED = 0xD64A0000

# RNG streams (see synth.c): 1 fanins, 2 inverters, 3 target levels.
STREAM_X = 4


def stream_wqkv(layer: int) -> int:
    return 100 + 3 * layer


def stream_wo(layer: int) -> int:
    return 101 + 3 * layer


def stream_bias(layer: int) -> int:
    return 102 + 3 * layer


def stream_w1(layer: int) -> int:
    return 200 + 2 * layer


def stream_w2(layer: int) -> int:
    return 201 + 2 * layer


@dataclass(frozen=True)
class Config:
    name: str
    index: int          # seed = BASE_SEED + index
    n_pi: int
    n_and: int
    window: int
    p_window: float     # 1.0: pair drawn without replacement from the window
    level_cap: int      # 0: none
    hidden: int
    heads: int
    hops: int
    n_layers: int
    dtype: str          # "f32" | "bf16"

    @property
    def n_nodes(self) -> int:
        return self.n_pi + self.n_and

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


CONFIGS = {
    "tiny":   Config("tiny",   0, 32,   1_000,     64,   1.0, 0,    128, 4, 2, 1, "f32"),
    "small":  Config("small",  1, 256,  20_000,    512,  1.0, 0,    128, 4, 2, 1, "f32"),
    "medium": Config("medium", 2, 1024, 200_000,   1024, 0.8, 0,    256, 8, 2, 1, "bf16"),
    "large":  Config("large",  3, 4096, 1_000_000, 1024, 0.8, 1000, 256, 8, 2, 1, "bf16"),
    "stress": Config("stress", 4, 8192, 4_000_000, 1024, 0.8, 1000, 256, 8, 3, 4, "bf16"),
}


def build(force: bool = False) -> str:
    """Compile synth.c with gcc into libdg4synth.so (in-tree)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"])
    return _SO


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.dg4s_rand.restype = ctypes.c_uint64
        lib.dg4s_rand.argtypes = [ctypes.c_uint64] * 3
        lib.dg4s_normal.restype = None
        lib.dg4s_normal.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int64,
                                    ctypes.c_double, ctypes.c_int32, ctypes.c_void_p]
        lib.dg4s_aig.restype = ctypes.c_int
        lib.dg4s_aig.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                 ctypes.c_double, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                 ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def rand_u64(seed: int, stream: int, i: int) -> int:
    return int(_load().dg4s_rand(seed, stream, i))


def normal(seed: int, stream: int, shape, scale: float = 1.0, bf16: bool = False) -> np.ndarray:
    """float32 array of N(0, scale^2) draws; bf16=True rounds each to bf16."""
    out = np.empty(shape, dtype=np.float32)
    _load().dg4s_normal(seed, stream, out.size, float(scale), int(bf16), out.ctypes.data)
    return out


def aig(seed: int, n_pi: int, n_and: int, window: int, p_window: float = 1.0, level_cap: int = 0):
    """(edge_src, edge_dst, edge_inv, level_hint|None); int32, int32, uint8, int32."""
    e = 2 * n_and
    src = np.empty(e, dtype=np.int32)
    dst = np.empty(e, dtype=np.int32)
    inv = np.empty(e, dtype=np.uint8)
    hint = np.empty(n_pi + n_and, dtype=np.int32) if level_cap > 0 else None
    rc = _load().dg4s_aig(seed, n_pi, n_and, window, float(p_window), level_cap,
                          src.ctypes.data, dst.ctypes.data, inv.ctypes.data,
                          hint.ctypes.data if hint is not None else None)
    if rc != 0:
        raise ValueError("dg4s_aig: bad arguments")
    return src, dst, inv, hint


def not_as_nodes(n: int, src, dst, inv):
    """The same circuit with inverters as NODES, the paper's own AIG form (Section 3.2: in-degree 1
    = NOT gate): every signal that some AND reads inverted gets ONE NOT node (structural hashing),
    id n + its rank among such signals, fed by a plain edge; the inverted edges into ANDs are
    re-attached to it as plain edges. Edges into in-degree-1 nodes are left alone.
    Returns (n2, src2, dst2, inv2, not_node) with not_node[v] = id of v's NOT node or -1."""
    src, dst, inv = (np.asarray(a) for a in (src, dst, inv))
    indeg = np.bincount(dst, minlength=n)
    moved = (inv == 1) & (indeg[dst] == 2)
    signals = np.unique(src[moved])
    not_node = np.full(n, -1, dtype=np.int32)
    not_node[signals] = n + np.arange(len(signals), dtype=np.int32)
    src2 = np.where(moved, not_node[src], src).astype(np.int32)
    inv2 = np.where(moved, 0, inv).astype(np.uint8)
    src2 = np.concatenate([src2, signals.astype(np.int32)])
    dst2 = np.concatenate([dst.astype(np.int32), not_node[signals]])
    inv2 = np.concatenate([inv2, np.zeros(len(signals), dtype=np.uint8)])
    return n + len(signals), src2, dst2, inv2, not_node


@dataclass
class Workload:
    cfg: Config
    edge_src: np.ndarray
    edge_dst: np.ndarray
    edge_inv: np.ndarray
    level_hint: np.ndarray | None
    x: np.ndarray                # [N, d] float32
    wqkv: list                   # per layer [d, 3d] float32, columns Q | K | V
    wo: list                     # per layer [d, d]
    rel_bias: list               # per layer [heads, 4] float32 (never rounded)


def weights(cfg: Config, seed: int | None = None):
    seed = cfg.seed if seed is None else seed
    bf = cfg.dtype == "bf16"
    d = cfg.hidden
    s = d ** -0.5                # variance 1/hidden
    wqkv = [normal(seed, stream_wqkv(l), (d, 3 * d), s, bf) for l in range(cfg.n_layers)]
    wo = [normal(seed, stream_wo(l), (d, d), s, bf) for l in range(cfg.n_layers)]
    rb = [normal(seed, stream_bias(l), (cfg.heads, 4), 1.0, False) for l in range(cfg.n_layers)]
    return wqkv, wo, rb


def ffn_weights(cfg: Config, seed: int | None = None):
    """Per layer W1 [d, 4d] ~ N(0, 1/d) and W2 [4d, d] ~ N(0, 1/(4d)) of the feed-forward sub-block."""
    seed = cfg.seed if seed is None else seed
    bf = cfg.dtype == "bf16"
    d = cfg.hidden
    w1 = [normal(seed, stream_w1(l), (d, 4 * d), d ** -0.5, bf) for l in range(cfg.n_layers)]
    w2 = [normal(seed, stream_w2(l), (4 * d, d), (4 * d) ** -0.5, bf) for l in range(cfg.n_layers)]
    return w1, w2


def make(cfg: Config | str, *, n_and: int | None = None, features: bool = True) -> Workload:
    """Build the workload of a configuration (optionally with fewer AND gates)."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    if n_and is not None:
        cfg = Config(**{**cfg.__dict__, "n_and": n_and})
    src, dst, inv, hint = aig(cfg.seed, cfg.n_pi, cfg.n_and, cfg.window, cfg.p_window, cfg.level_cap)
    bf = cfg.dtype == "bf16"
    x = normal(cfg.seed, STREAM_X, (cfg.n_nodes, cfg.hidden), 1.0, bf) if features else None
    wqkv, wo, rb = weights(cfg)
    return Workload(cfg, src, dst, inv, hint, x, wqkv, wo, rb)
