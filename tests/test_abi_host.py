"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, reports the flat layout the workloads use, and rejects bad arguments before
anything is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2009_02701_amd import binding as hb
from paper_2009_02701_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "hpsgd.h")).read()
    declared = set(re.findall(r"\b(hpsgd_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(hb.EXPORTS), declared ^ set(hb.EXPORTS)
    lib = C.CDLL(hb.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


@pytest.mark.parametrize("name", ["tiny_gru", "gru_cls", "gru_lm", "mlp"])
def test_flat_layout_matches_workload_shapes(name):
    cfg = wl.CONFIGS[name]
    ctx = hb.Context(cfg)
    shapes = wl.param_shapes(cfg)
    assert ctx.P == wl.param_count(cfg)
    assert [e[0] for e in ctx.entries] == [n for n, _ in shapes]
    off = 0
    for (n, o, rows, cols), (_, shp) in zip(ctx.entries, shapes):
        assert o == off and rows * cols == int(np.prod(shp)) and rows == shp[0]
        off += rows * cols
    assert ctx.workspace_bytes > 4 * ctx.P * ctx.K


def test_param_counts_of_the_five_configs():
    assert hb.Context(wl.CONFIGS["tiny_gru"]).P == 5130
    assert hb.Context(wl.CONFIGS["gru_cls"]).P == 991242
    assert hb.Context(wl.CONFIGS["gru_lm"]).P == 23045904
    assert hb.Context(wl.CONFIGS["mlp"]).P == 1863690


def test_flatten_roundtrip():
    cfg = wl.CONFIGS["tiny_gru"]
    ctx = hb.Context(cfg)
    p = wl.init_params(cfg)
    back = ctx.unflatten(ctx.flatten(p))
    for k in p:
        assert back[k].shape == p[k].shape and np.array_equal(back[k], p[k])


def test_create_rejects_bad_descriptions():
    lib = hb.load_library()
    h = C.c_void_p()
    good = hb.make_desc(wl.CONFIGS["tiny_gru"])
    assert lib.hpsgd_create(C.byref(good), 0, C.byref(h)) == 1          # K < 1
    assert lib.hpsgd_create(C.byref(good), 33, C.byref(h)) == 1         # K > max
    assert lib.hpsgd_create(None, 2, C.byref(h)) == 1
    bad = hb.make_desc(wl.scaled(wl.CONFIGS["tiny_gru"], hidden=0))
    assert lib.hpsgd_create(C.byref(bad), 2, C.byref(h)) == 2           # shape
    bad = hb.make_desc(wl.scaled(wl.CONFIGS["mlp"], dims=[5]))
    assert lib.hpsgd_create(C.byref(bad), 2, C.byref(h)) == 2
    bad = hb.make_desc(wl.CONFIGS["tiny_gru"])
    bad.kind = 9
    assert lib.hpsgd_create(C.byref(bad), 2, C.byref(h)) == 1
    assert not h.value


def test_merge_and_sync_reject_bad_arguments_before_launch():
    """Fake (never dereferenced) addresses: every call must fail in validation."""
    lib = hb.load_library()
    vp = C.c_void_p
    A, B, S = 0x10000, 0x20000, 0x30000
    reps = (vp * 2)(B, B + 0x8000)
    assert lib.hpsgd_merge(vp(A), reps, vp(S), 0, 16, None) == 1         # K < 1
    assert lib.hpsgd_merge(vp(A), reps, vp(S), 40, 16, None) == 1        # K > max
    assert lib.hpsgd_merge(None, reps, vp(S), 2, 16, None) == 1          # null
    assert lib.hpsgd_merge(vp(A), None, vp(S), 2, 16, None) == 1
    assert lib.hpsgd_merge(vp(A + 4), reps, vp(S), 2, 16, None) == 3     # misaligned
    bad = (vp * 2)(B, A + 16)
    assert lib.hpsgd_merge(vp(A), bad, vp(S), 2, 16, None) == 4          # replica overlaps global
    assert lib.hpsgd_merge(vp(A), reps, vp(A + 16), 2, 16, None) == 4    # partial snapshot overlap
    assert lib.hpsgd_merge(vp(A), reps, vp(S), 2, 0, None) == 0          # empty: no-op
    assert lib.hpsgd_sync_all(vp(A), reps, 2, vp(A), 16, None) == 4
    assert lib.hpsgd_sync_all(vp(A), reps, 2, vp(S + 8), 16, None) == 3
    assert lib.hpsgd_sync_replica(vp(A), None, 16, None) == 1
    assert lib.hpsgd_sync_replica(vp(A), vp(A), 16, None) == 4
    assert lib.hpsgd_gather_batch(vp(A), vp(B), 4, 6, 1, 4, vp(S), None) == 3   # row bytes not /4
    assert lib.hpsgd_gather_batch(vp(A), vp(B), 4, 8, 3, 4, vp(S), None) == 2   # chunks exceed row
    assert lib.hpsgd_gather_batch(vp(A), vp(B), -1, 8, 1, 4, vp(S), None) == 1


def test_gather_all_and_aux_stream_reject_bad_arguments():
    lib = hb.load_library()
    vp = C.c_void_p
    sh = (vp * 2)(0x10000, 0x20000)
    ix = (vp * 2)(0x30000, 0x40000)
    out = (vp * 2)(0x50000, 0x60000)
    call = lib.hpsgd_gather_batch_all
    assert call(sh, ix, 40, 4, 8, 1, 8, out, None) == 1                  # K > max
    assert call(sh, ix, 2, -1, 8, 1, 8, out, None) == 1
    assert call(None, ix, 2, 4, 8, 1, 8, out, None) == 1
    assert call(sh, ix, 2, 4, 6, 1, 4, out, None) == 3                   # row bytes not a multiple of 4
    assert call(sh, ix, 2, 4, 8, 3, 4, out, None) == 2                   # chunks exceed the row
    bad = (vp * 2)(0x10000, 0)
    assert call(bad, ix, 2, 4, 8, 1, 8, out, None) == 1                  # null shard pointer
    bad = (vp * 2)(0x10000, 0x20002)
    assert call(bad, ix, 2, 4, 8, 1, 8, out, None) == 3                  # misaligned shard pointer
    assert call(sh, ix, 0, 4, 8, 1, 8, out, None) == 0                   # no workers: no-op
    assert lib.hpsgd_set_aux_stream(None, None) == 1
    ctx = hb.Context(wl.CONFIGS["tiny_gru"])
    assert lib.hpsgd_set_aux_stream(ctx._h, None) == 0                   # switching it off needs no GPU
    assert lib.hpsgd_timer_enable(None, 0) == 1
    assert lib.hpsgd_timer_read(ctx._h, 99, None, None) == 1
    assert lib.hpsgd_role_name(99) is None and lib.hpsgd_role_name(3) == b"gemm_recurrent_bwd"
    assert lib.hpsgd_commit_kernel_params(None) == 0 and lib.hpsgd_commit_kernel_params(ctx._h) == 0
    mg = lib.hpsgd_merge_grad
    ok = (vp * 2)(0x1000, 0x2000)
    assert mg(0x10000, ok, 0.1, 0, 64, None) == 1                        # K < 1
    assert mg(0x10000, ok, 0.1, 2, 0, None) == 0                         # P == 0: no-op
    assert mg(None, ok, 0.1, 2, 64, None) == 1
    assert mg(0x10004, ok, 0.1, 2, 64, None) == 3                        # misaligned global
    assert mg(0x10000, (vp * 2)(0x1000, 0x2004), 0.1, 2, 64, None) == 3  # misaligned accumulator
    assert mg(0x1000, ok, 0.1, 2, 64, None) == 4                         # accumulator aliases global
    assert lib.hpsgd_local_step_all_acc(None, 0x1000, 0x1000, 64, 0x2000, 0x3000, 0.1, None, 0x4000, 64,
                                        0x5000, None) == 1
    assert lib.hpsgd_set_recurrence(None, 1, 100) == 1
    assert lib.hpsgd_set_recurrence(ctx._h, 0, 0) == 0 and lib.hpsgd_set_recurrence(ctx._h, 1, 1 << 20) == 0
    gave, n0, n1, n2 = C.c_int(7), C.c_int(7), C.c_int(7), C.c_int(7)
    assert lib.hpsgd_recurrence_gave_up(None, 0x1000, None, C.byref(gave)) == 1
    assert lib.hpsgd_recurrence_gave_up(ctx._h, 0x1000, None, None) == 1
    assert lib.hpsgd_recurrence_gave_up(ctx._h, None, None, C.byref(gave)) == 5      # no workspace
    assert lib.hpsgd_recurrence_info(None, C.byref(n0), C.byref(n1), C.byref(n2)) == 1
    assert lib.hpsgd_recurrence_info(ctx._h, C.byref(n0), None, C.byref(n2)) == 0    # before any step: zeros
    assert (n0.value, n1.value, n2.value) == (0, 7, 0)
    assert lib.hpsgd_delay_us(2000000, None) == 1                        # beyond the one-second cap
    assert lib.hpsgd_delay_us(0, None) == 0                              # nothing to launch
    probe = lib.hpsgd_probe_mfma_rate
    assert probe(0, None, 10, 0x1000, 0x2000, None) == 1                 # null operands
    assert probe(0, 0x1000, 0, 0x2000, 0x3000, None) == 1                # no iterations
    assert probe(7, 0x1000, 10, 0x2000, 0x3000, None) == 1               # unknown precision
    assert probe(1, 0x1004, 10, 0x2000, 0x3000, None) == 3               # misaligned operands


def test_local_step_rejects_bad_arguments_before_launch():
    lib = hb.load_library()
    ctx = hb.Context(wl.CONFIGS["tiny_gru"])
    vp = C.c_void_p
    R, O, X, Y, W = 0x100000, 0x200000, 0x300000, 0x400000, 0x1000000
    call = lambda r, o, stride, x, y, w: lib.hpsgd_local_step_all(ctx._h, vp(r), vp(o), stride, vp(x), vp(y),
                                                                   0.1, None, vp(w), None)
    assert call(0, O, 5132, X, Y, W) == 1
    assert call(R, O, 5132, X, Y, 0) == 5
    assert call(R, O, 5132, X, Y, W + 16) == 5
    assert call(R + 4, O, 5132, X, Y, W) == 3
    assert call(R, O, 5130, X, Y, W) == 3                                # stride not a multiple of 4
    assert call(R, O, 5000, X, Y, W) == 3                                # stride < P
    assert call(R, R + 64, 5132, X, Y, W) == 4                           # partial overlap in/out
    assert call(R, O, 5132, X, Y, R) == 4                                # workspace over the replicas
    assert lib.hpsgd_local_step(ctx._h, 2, vp(R), vp(O), vp(X), vp(Y), 0.1, None, vp(W), None) == 1
    prep = lambda r, stride, w: lib.hpsgd_prepare_replicas(ctx._h, vp(r), stride, vp(w), None)
    assert prep(0, 5132, W) == 1
    assert prep(R, 5132, 0) == 5 and prep(R, 5132, W + 16) == 5
    assert prep(R + 4, 5132, W) == 3 and prep(R, 5130, W) == 3 and prep(R, 5000, W) == 3
    assert prep(R, 5132, R) == 4
    assert prep(R, 5132, W) == 0                                         # fp32: nothing to prepare, nothing launched
    assert hb.load_library().hpsgd_strerror(4) == b"buffers overlap"
    # clone + step as one call: the source is one model of P floats beside the K output replicas
    G = 0x080000
    cl = lambda g, o, stride, x, y, w: lib.hpsgd_local_step_all_cloned(ctx._h, vp(g), vp(o), stride, vp(x), vp(y),
                                                                      0.1, None, vp(w), None)
    assert lib.hpsgd_local_step_all_cloned(None, vp(G), vp(O), 5132, vp(X), vp(Y), 0.1, None, vp(W), None) == 1
    assert cl(0, O, 5132, X, Y, W) == 1                                   # no source
    assert cl(G, 0, 5132, X, Y, W) == 1                                   # no output
    assert cl(G + 4, O, 5132, X, Y, W) == 3                               # misaligned source
    assert cl(G, O, 5130, X, Y, W) == 3 and cl(G, O, 5000, X, Y, W) == 3  # output stride
    assert cl(O, O, 5132, X, Y, W) == 4                                   # the source is a replica being written
    assert cl(O + 4 * 5132, O, 5132, X, Y, W) == 4                        # ... any of them
    assert cl(W + 256, O, 5132, X, Y, W) == 4                             # the source inside the workspace
    assert cl(G, O, 5132, X, Y, 0) == 5


def test_kernel_timer_entry_points_on_the_host():
    """hpsgd_kernel_name covers ids 1 .. HPSGD_KERNEL_COUNT-1 (the enum of the header), and the
    timer calls check their arguments; nothing here launches."""
    lib = hb.load_library()
    hdr = open(os.path.join(ROOT, "include", "hpsgd.h")).read()
    count = int(re.search(r"HPSGD_KERNEL_COUNT = (\d+)", hdr).group(1))
    assert count == hb.KERNEL_COUNT
    names = [lib.hpsgd_kernel_name(i) for i in range(count)]
    assert names[0] is None and all(n for n in names[1:]) and len(set(names[1:])) == count - 1
    assert lib.hpsgd_kernel_name(count) is None and lib.hpsgd_kernel_name(-1) is None
    ctx = hb.Context(wl.CONFIGS["tiny_gru"])
    assert lib.hpsgd_kernel_timer_enable(None, 1) == 1
    assert lib.hpsgd_kernel_timer_enable(ctx._h, 0xFFFFFFFF) == 0
    n, ms, w = C.c_long(-1), C.c_double(-1), C.c_double(-1)
    assert lib.hpsgd_kernel_timer_read(ctx._h, 0, C.byref(n), C.byref(ms), C.byref(w)) == 1
    assert lib.hpsgd_kernel_timer_read(ctx._h, count, C.byref(n), C.byref(ms), C.byref(w)) == 1
    assert lib.hpsgd_kernel_timer_read(ctx._h, 1, C.byref(n), C.byref(ms), C.byref(w)) == 0
    assert n.value == 0 and ms.value == 0.0 and w.value == 0.0
    assert ctx.kernel_names()[4] == "gru_bwd_persist_bf16_kernel"


def test_static_workspace_entry_point_checks_the_size_before_any_device():
    """hpsgd_local_step_all_static refuses a model whose workspace exceeds its fixed array; the
    check needs no GPU.  The limit is the header's."""
    lib = hb.load_library()
    hdr = open(os.path.join(ROOT, "include", "hpsgd.h")).read()
    assert re.search(r"#define HPSGD_STATIC_WORKSPACE_BYTES \(32u << 20\)", hdr)
    ctx = hb.Context(wl.CONFIGS["gru_cls"])
    assert ctx.workspace_bytes > (32 << 20)
    dummy = C.c_void_p(4096)
    assert lib.hpsgd_local_step_all_static(ctx._h, dummy, dummy, C.c_size_t(ctx.stride), dummy, dummy,
                                           C.c_float(0.1), None, None) == 5
    assert lib.hpsgd_local_step_all_static(None, dummy, dummy, C.c_size_t(4), dummy, dummy, C.c_float(0.1), None,
                                           None) == 1


def test_merge_sync_checks_its_arguments_on_the_host():
    lib = hb.load_library()
    P = 64
    a = lambda i: C.c_void_p(0x10000 + 0x1000 * i)
    reps = (C.c_void_p * 2)(a(2), a(3))
    assert lib.hpsgd_merge_sync(a(0), reps, a(1), 0, P, None) == 1                      # K < 1
    assert lib.hpsgd_merge_sync(None, reps, a(1), 2, P, None) == 1                      # null
    assert lib.hpsgd_merge_sync(a(0), reps, a(1), 2, 0, None) == 0                      # empty: no-op
    assert lib.hpsgd_merge_sync(C.c_void_p(0x10004), reps, a(1), 2, P, None) == 3       # alignment
    assert lib.hpsgd_merge_sync(a(0), reps, a(0), 2, P, None) == 4                      # snapshot == global
    same = (C.c_void_p * 2)(a(2), a(2))
    assert lib.hpsgd_merge_sync(a(0), same, a(1), 2, P, None) == 4                      # a replica twice
    onto = (C.c_void_p * 2)(a(2), a(1))
    assert lib.hpsgd_merge_sync(a(0), onto, a(1), 2, P, None) == 4                      # replica == snapshot
    # merge + snapshot in one pass: the replicas are only read (one may be passed twice)
    ms = lib.hpsgd_merge_snapshot
    assert ms(a(0), reps, a(1), 0, P, None) == 1 and ms(None, reps, a(1), 2, P, None) == 1
    assert ms(a(0), reps, None, 2, P, None) == 1
    assert ms(a(0), reps, a(1), 2, 0, None) == 0
    assert ms(C.c_void_p(0x10004), reps, a(1), 2, P, None) == 3
    assert ms(a(0), reps, a(0), 2, P, None) == 4                                        # snapshot == global
    assert ms(a(0), onto, a(1), 2, P, None) == 4                                        # replica == snapshot
    assert ms(a(2), reps, a(1), 2, P, None) == 4                                        # replica == global


def test_prepare_clones_checks_its_arguments_on_the_host():
    lib = hb.load_library()
    ctx = hb.Context(wl.CONFIGS["tiny_gru"])   # fp32: nothing to prepare, but the arguments are checked
    a = lambda i: C.c_void_p(0x100000 + 0x10000 * i)
    ws = C.c_void_p(0x4000000)
    assert lib.hpsgd_prepare_clones(None, a(0), a(1), C.c_size_t(ctx.stride), ws, 0, None) == 1
    assert lib.hpsgd_prepare_clones(ctx._h, None, a(1), C.c_size_t(ctx.stride), ws, 0, None) == 1
    assert lib.hpsgd_prepare_clones(ctx._h, a(0), a(1), C.c_size_t(ctx.stride), None, 0, None) == 5
    assert lib.hpsgd_prepare_clones(ctx._h, a(0), a(1), C.c_size_t(ctx.stride), C.c_void_p(0x4000010), 0, None) == 5
    assert lib.hpsgd_prepare_clones(ctx._h, C.c_void_p(0x100004), a(1), C.c_size_t(ctx.stride), ws, 0, None) == 3
    assert lib.hpsgd_prepare_clones(ctx._h, a(0), a(1), C.c_size_t(ctx.P - 1), ws, 0, None) == 3   # stride < P
    assert lib.hpsgd_prepare_clones(ctx._h, a(0), a(1), C.c_size_t(ctx.stride), a(1), 0, None) == 4  # workspace on the replicas
    assert lib.hpsgd_prepare_clones(ctx._h, a(0), a(1), C.c_size_t(ctx.stride), ws, 0, None) == 0
