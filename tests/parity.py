"""Shared helpers of the GPU parity tests (no arithmetic of the method)."""
import numpy as np

from oracle import hpsgd_oracle as oc
from paper_2009_02701_amd import workloads as wl

# spec tolerances: max relative error per tensor, ||gpu - ref||_inf / ||ref||_inf
TOL_FP32 = 1e-4
TOL_BF16 = 2e-2


def rel_err(got, want) -> float:
    want = np.asarray(want, np.float64)
    got = np.asarray(got, np.float64)
    scale = np.abs(want).max()
    if scale == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - want).max() / scale)


def worst_rel_err(got: dict, want: dict):
    assert set(got) == set(want)
    errs = {k: rel_err(got[k], want[k]) for k in want}
    k = max(errs, key=errs.get)
    return errs[k], k, errs


def workload(cfg):
    K = cfg["K"]
    init = wl.init_params(cfg)
    shards = [wl.make_shard(cfg, k) for k in range(K)]
    orders = [wl.batch_order(cfg, k) for k in range(K)]
    batch_fn = lambda k, s: oc.gather_batch(cfg["kind"], shards[k][0], shards[k][1], wl.batch_indices(cfg, k, s))
    return init, shards, orders, batch_fn


def round_bf16(a):
    """Round-to-nearest-even to bfloat16 (8 significand bits), returned as float64.
    Pinned in tests/test_oracle_model.py against the library's conversion and hand-written ties."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)
