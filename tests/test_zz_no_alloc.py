"""dg4_qkv_proj_static (the entry point for callers that cannot allocate) against dg4_qkv_proj.

Collected last: the scratch array inside the library is shared by every call on the GPU, so this
file also checks that nothing of an earlier call's contents leaks into a later, smaller one.
"""
import ctypes

import numpy as np
import pytest
import torch

import dg4_synth as synth
import oracle
import paper_2502_01681_amd as dg4
from gpu_utils import TOL, row_rel_err, tdtype, to_dev, to_np


def test_static_rejects_what_does_not_fit():
    # fp32 with hidden 256 packs into 768 KB: more than the array. Turned away before any device call.
    assert dg4.dg4_static_scratch_bytes() == 512 * 1024
    cfg = dg4.LayerConfig(256, 8, 2, 1, "f32")
    assert dg4.dg4_proj_workspace_bytes(cfg) > dg4.dg4_static_scratch_bytes()
    c = cfg.c()
    fake = ctypes.c_void_p(4096)          # non-null, aligned; never dereferenced
    rc = dg4.lib().dg4_qkv_proj_static(ctypes.byref(c), fake, 0, 8, fake, fake, fake, fake, None)
    assert rc == -8                        # DG4_EWORKSPACE
    rc = dg4.lib().dg4_qkv_proj_static(ctypes.byref(c), None, 0, 8, fake, fake, fake, fake, None)
    assert rc == -1                        # DG4_EINVAL comes first


def _both(dtype, d, rows, lo, hi, seed):
    bf = dtype == "bf16"
    S = synth.normal(seed, 4, (rows, d), 1.0, bf)
    W = synth.normal(seed, 100, (d, 3 * d), d ** -0.5, bf)
    cfg = dg4.LayerConfig(d, d // 32, 2, 1, dtype)
    Sd, Wd = to_dev(S, dtype), to_dev(W, dtype)
    ref = [torch.full((rows, d), 7.0, dtype=tdtype(dtype), device="cuda") for _ in range(3)]
    got = [torch.full((rows, d), 7.0, dtype=tdtype(dtype), device="cuda") for _ in range(3)]
    dg4.dg4_qkv_proj(cfg, Sd, Wd, *ref, row_begin=lo, row_end=hi)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    dg4.dg4_qkv_proj_static(cfg, Sd, Wd, *got, row_begin=lo, row_end=hi)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    orc = oracle.qkv_proj(S, W)
    for a, b, r in zip(got, ref, orc):
        assert torch.equal(a, b)                                         # same kernels: bit for bit
        a = to_np(a)
        assert (a[:lo] == 7.0).all() and (a[hi:] == 7.0).all()
        if hi > lo:
            assert row_rel_err(a[lo:hi], r[lo:hi]).max() <= TOL[dtype]   # and the oracle's bar


@pytest.mark.gpu
def test_static_matches_workspace_call_twice_in_a_row():
    print("qkv_proj_static bf16 d=256 rows=4133 then f32 d=128 rows=77", flush=True)
    _both("bf16", 256, 4133, 5, 4100, 51)         # several tiles, ragged tail, fills 384 KB of the array
    _both("f32", 128, 77, 3, 77, 52)              # smaller input, smaller packed weight (192 KB), other kernels
    _both("bf16", 128, 300, 0, 300, 53)           # 96 KB
    _both("bf16", 256, 64, 0, 33, 54)             # back to the large weight, few rows


@pytest.mark.gpu
def test_static_empty_range_touches_nothing():
    cfg = dg4.LayerConfig(128, 4, 2, 1, "f32")
    t = torch.zeros((4, 128), device="cuda")
    w = torch.zeros((128, 384), device="cuda")
    dg4.dg4_qkv_proj_static(cfg, t, w, t, t, t, row_begin=2, row_end=2)
    torch.cuda.synchronize()
