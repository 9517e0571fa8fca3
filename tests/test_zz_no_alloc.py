"""hpsgd_local_step_all_static: the entry point that allocates nothing, through the C ABI,
against hpsgd_local_step_all on the same inputs."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2009_02701_amd import binding as hb
from paper_2009_02701_amd import harness
from paper_2009_02701_amd import workloads as wl

from parity import workload

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

BIG = wl.scaled(wl.CONFIGS["gru_lm"], vocab=264, embed=72, hidden=160, seq_len=19, batch=16, K=2)   # 17 MiB, bf16
SMALL = wl.CONFIGS["tiny_gru"]                                                                     # 0.24 MiB, fp32


def _both_entry_points(cfg, steps=2):
    """`steps` local steps through each entry point, raw C-ABI calls; returns (replicas, losses) of both."""
    init, shards, orders, _ = workload(cfg)
    tr = harness.Trainer(cfg, init, shards, orders, device=DEV)
    lib, ctx = hb.load_library(), tr.ctx
    assert ctx.workspace_bytes <= (32 << 20)
    tr.sync_all(0)
    tr.sync_all(1)
    torch.cuda.synchronize()
    st = torch.cuda.current_stream()
    out = []
    for gen, static in ((0, False), (1, True)):
        R = tr.R[gen]
        loss = torch.zeros(steps, cfg["K"], device=DEV)
        for i in range(steps):
            tr.gather(i)
            args = [ctx._h, C.c_void_p(R.data_ptr()), C.c_void_p(R.data_ptr()), C.c_size_t(R.stride(0)),
                    C.c_void_p(tr.xb.data_ptr()), C.c_void_p(tr.yb.data_ptr()), C.c_float(cfg["lr"]),
                    C.c_void_p(loss[i].data_ptr())]
            if static:
                rc = lib.hpsgd_local_step_all_static(*args, C.c_void_p(st.cuda_stream))
            else:
                rc = lib.hpsgd_local_step_all(*args, ctx._ws_ptr(tr.ws[0]), C.c_void_p(st.cuda_stream))
            assert rc == 0, rc
        torch.cuda.synchronize()
        out.append((R[:, :tr.P].clone(), loss.clone()))
    return out


def test_static_workspace_entry_point_twice_in_a_row_second_call_smaller():
    """Two uses in a row, the second with a smaller model (the array then still holds the first
    one's contents): each gives the bits of hpsgd_local_step_all, losses included."""
    for cfg in (BIG, SMALL, BIG):
        (r0, l0), (r1, l1) = _both_entry_points(cfg)
        assert torch.isfinite(r0).all() and torch.isfinite(l0).all()
        assert torch.equal(r0, r1), cfg
        assert torch.equal(l0, l1), cfg


def test_static_workspace_entry_point_rejects_models_beyond_its_array():
    cfg = wl.CONFIGS["gru_cls"]   # 276 MiB of workspace
    ctx = hb.Context(cfg)
    lib = hb.load_library()
    R = torch.zeros(cfg["K"], ctx.stride, device=DEV)
    x = torch.zeros(cfg["K"], cfg["seq_len"], cfg["batch"], cfg["input"], device=DEV)
    y = torch.zeros(cfg["K"], cfg["batch"], dtype=torch.int32, device=DEV)
    rc = lib.hpsgd_local_step_all_static(ctx._h, C.c_void_p(R.data_ptr()), C.c_void_p(R.data_ptr()),
                                         C.c_size_t(R.stride(0)), C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr()),
                                         C.c_float(0.1), None, None)
    assert rc == 5  # HPSGD_EWORKSPACE
    assert float(R.abs().sum()) == 0.0
