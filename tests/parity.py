"""Shared helpers of the GPU parity tests (no arithmetic of the method)."""
import numpy as np

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
    batch_fn = lambda k, s: wl.host_batch(cfg, shards[k], wl.batch_indices(cfg, k, s))
    return init, shards, orders, batch_fn


def round_bf16(a):
    """Round-to-nearest-even to bfloat16 (8 significand bits), returned as float64."""
    u = np.asarray(a, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)
