"""ctypes binding of libhpsgd.so: argument marshalling only.

Every arithmetic step of the hot path runs in the library's HIP kernels; torch tensors
are used for device memory and streams.  If the shared library is missing or a call
returns an error code this module raises -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhpsgd.so")

KIND = {"gru_cls": 0, "gru_lm": 1, "mlp": 2}
PREC = {"fp32": 0, "bf16": 1}
MAX_MLP_DIMS = 8

EXPORTS = [
    "hpsgd_create", "hpsgd_destroy", "hpsgd_param_count", "hpsgd_param_entries",
    "hpsgd_param_entry", "hpsgd_workspace_bytes", "hpsgd_local_step_all", "hpsgd_local_step",
    "hpsgd_gather_batch", "hpsgd_gather_batch_all", "hpsgd_merge", "hpsgd_sync_replica", "hpsgd_sync_all", "hpsgd_strerror",
    "hpsgd_set_aux_stream", "hpsgd_timer_enable", "hpsgd_timer_read", "hpsgd_role_name",
    "hpsgd_commit_kernel_params", "hpsgd_probe_mfma_rate", "hpsgd_delay_us",
    "hpsgd_local_step_all_acc", "hpsgd_merge_grad", "hpsgd_set_recurrence", "hpsgd_recurrence_gave_up",
    "hpsgd_recurrence_info", "hpsgd_gemm_bf16_nt", "hpsgd_prepare_replicas",
    "hpsgd_kernel_timer_enable", "hpsgd_kernel_timer_read", "hpsgd_kernel_name",
    "hpsgd_local_step_all_static", "hpsgd_local_step_all_cloned", "hpsgd_merge_sync", "hpsgd_merge_snapshot", "hpsgd_prepare_clones",
]
ROLE_COUNT = 14
KERNEL_COUNT = 22


class ModelDesc(C.Structure):
    _fields_ = [("kind", C.c_int), ("prec", C.c_int), ("layers", C.c_int), ("input", C.c_int),
                ("hidden", C.c_int), ("seq_len", C.c_int), ("batch", C.c_int), ("classes", C.c_int),
                ("vocab", C.c_int), ("embed", C.c_int), ("n_mlp_dims", C.c_int),
                ("mlp_dims", C.c_int * MAX_MLP_DIMS)]


class HpsgdError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: {code}")
        self.code = code


_lib = None


def load_library():
    """Load libhpsgd.so (built in-tree by __graft_entry__.build()); raise if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(LIB_PATH)
    vp, sz, i32p = C.c_void_p, C.c_size_t, C.c_void_p
    lib.hpsgd_create.argtypes = [C.POINTER(ModelDesc), C.c_int, C.POINTER(vp)]
    lib.hpsgd_destroy.argtypes = [vp]
    lib.hpsgd_param_count.argtypes = [vp]
    lib.hpsgd_param_count.restype = sz
    lib.hpsgd_param_entries.argtypes = [vp]
    lib.hpsgd_param_entry.argtypes = [vp, C.c_int, C.POINTER(C.c_char_p), C.POINTER(sz),
                                      C.POINTER(C.c_int), C.POINTER(C.c_int)]
    lib.hpsgd_workspace_bytes.argtypes = [vp]
    lib.hpsgd_workspace_bytes.restype = sz
    lib.hpsgd_local_step_all.argtypes = [vp, vp, vp, sz, vp, i32p, C.c_float, vp, vp, vp]
    lib.hpsgd_local_step_all_cloned.argtypes = [vp, vp, vp, sz, vp, i32p, C.c_float, vp, vp, vp]
    lib.hpsgd_local_step_all_static.argtypes = [vp, vp, vp, sz, vp, i32p, C.c_float, vp, vp]
    lib.hpsgd_prepare_replicas.argtypes = [vp, vp, sz, vp, vp]
    lib.hpsgd_prepare_clones.argtypes = [vp, vp, vp, sz, vp, C.c_int, vp]
    lib.hpsgd_local_step.argtypes = [vp, C.c_int, vp, vp, vp, i32p, C.c_float, vp, vp, vp]
    lib.hpsgd_gather_batch.argtypes = [vp, i32p, C.c_int, sz, C.c_int, sz, vp, vp]
    lib.hpsgd_gather_batch_all.argtypes = [C.POINTER(vp), C.POINTER(vp), C.c_int, C.c_int, sz, C.c_int, sz,
                                           C.POINTER(vp), vp]
    lib.hpsgd_merge.argtypes = [vp, C.POINTER(vp), vp, C.c_int, sz, vp]
    lib.hpsgd_merge_sync.argtypes = [vp, C.POINTER(vp), vp, C.c_int, sz, vp]
    lib.hpsgd_merge_snapshot.argtypes = [vp, C.POINTER(vp), vp, C.c_int, sz, vp]
    lib.hpsgd_sync_replica.argtypes = [vp, vp, sz, vp]
    lib.hpsgd_sync_all.argtypes = [vp, C.POINTER(vp), C.c_int, vp, sz, vp]
    lib.hpsgd_set_aux_stream.argtypes = [vp, vp]
    lib.hpsgd_set_recurrence.argtypes = [vp, C.c_int, C.c_uint]
    lib.hpsgd_recurrence_gave_up.argtypes = [vp, vp, vp, C.POINTER(C.c_int)]
    lib.hpsgd_recurrence_info.argtypes = [vp, C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int)]
    lib.hpsgd_timer_enable.argtypes = [vp, C.c_uint]
    lib.hpsgd_timer_read.argtypes = [vp, C.c_int, C.POINTER(C.c_long), C.POINTER(C.c_double)]
    lib.hpsgd_role_name.argtypes = [C.c_int]
    lib.hpsgd_role_name.restype = C.c_char_p
    lib.hpsgd_kernel_timer_enable.argtypes = [vp, C.c_uint]
    lib.hpsgd_kernel_timer_read.argtypes = [vp, C.c_int, C.POINTER(C.c_long), C.POINTER(C.c_double),
                                            C.POINTER(C.c_double)]
    lib.hpsgd_kernel_name.argtypes = [C.c_int]
    lib.hpsgd_kernel_name.restype = C.c_char_p
    lib.hpsgd_commit_kernel_params.argtypes = [vp]
    lib.hpsgd_commit_kernel_params.restype = sz
    lib.hpsgd_probe_mfma_rate.argtypes = [C.c_int, vp, C.c_int, vp, vp, vp]
    lib.hpsgd_delay_us.argtypes = [C.c_uint, vp]
    lib.hpsgd_gemm_bf16_nt.argtypes = [vp, C.c_long, C.c_long, vp, C.c_long, C.c_long, vp, C.c_long, C.c_long, vp,
                                       C.c_long, C.c_float, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, vp]
    lib.hpsgd_local_step_all_acc.argtypes = [vp, vp, vp, sz, vp, i32p, C.c_float, vp, vp, sz, vp, vp]
    lib.hpsgd_merge_grad.argtypes = [vp, C.POINTER(vp), C.c_float, C.c_int, sz, vp]
    lib.hpsgd_strerror.argtypes = [C.c_int]
    lib.hpsgd_strerror.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc, what):
    if rc != 0:
        raise HpsgdError(f"{rc} ({load_library().hpsgd_strerror(rc).decode()})", what)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr() if t is not None else None)


def make_desc(cfg: dict) -> ModelDesc:
    d = ModelDesc()
    d.kind = KIND[cfg["kind"]]
    d.prec = PREC[cfg.get("prec", "fp32")]
    for f in ("layers", "input", "hidden", "seq_len", "batch", "classes", "vocab", "embed"):
        setattr(d, f, int(cfg.get(f, 0)))
    dims = cfg.get("dims", [])
    d.n_mlp_dims = len(dims)
    for i, v in enumerate(dims[:MAX_MLP_DIMS]):
        d.mlp_dims[i] = int(v)
    return d


class Context:
    """hpsgd_ctx: the model every worker trains, K workers, flat layout and workspace size."""

    def __init__(self, cfg: dict, K: int | None = None):
        self.lib = load_library()
        self.cfg = dict(cfg)
        self.K = int(cfg["K"] if K is None else K)
        self._h = C.c_void_p()
        desc = make_desc(cfg)
        _check(self.lib.hpsgd_create(C.byref(desc), self.K, C.byref(self._h)), "hpsgd_create")
        self.P = int(self.lib.hpsgd_param_count(self._h))
        self.stride = (self.P + 3) // 4 * 4
        self.entries = []
        for i in range(self.lib.hpsgd_param_entries(self._h)):
            name, off, rows, cols = C.c_char_p(), C.c_size_t(), C.c_int(), C.c_int()
            _check(self.lib.hpsgd_param_entry(self._h, i, C.byref(name), C.byref(off), C.byref(rows),
                                              C.byref(cols)), "hpsgd_param_entry")
            self.entries.append((name.value.decode(), int(off.value), int(rows.value), int(cols.value)))
        self.workspace_bytes = int(self.lib.hpsgd_workspace_bytes(self._h))

    def __del__(self):
        if getattr(self, "_h", None) and self._h.value:
            self.lib.hpsgd_destroy(self._h)
            self._h = C.c_void_p()

    # ---- flat layout helpers (host side, numpy) ----
    def flatten(self, params: dict) -> np.ndarray:
        flat = np.zeros(self.P, np.float32)
        for name, off, rows, cols in self.entries:
            flat[off:off + rows * cols] = np.asarray(params[name], np.float32).reshape(-1)
        return flat

    def unflatten(self, flat) -> dict:
        flat = np.asarray(flat)
        out = {}
        for name, off, rows, cols in self.entries:
            v = flat[off:off + rows * cols]
            out[name] = v.reshape(rows, cols) if cols > 1 or name.endswith((".W", ".W_ih", ".W_hh", ".E")) \
                else v.reshape(rows)
        return out

    def new_workspace(self, device="cuda"):
        return torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=device)

    @staticmethod
    def _ws_ptr(ws):
        p = ws.data_ptr()
        return C.c_void_p((p + 255) // 256 * 256)

    def set_aux_stream(self, stream):
        """Second stream for the weight-gradient GEMMs that can run beside the recurrence (None = off)."""
        self._aux = stream  # keep the torch stream alive
        _check(self.lib.hpsgd_set_aux_stream(self._h, C.c_void_p(stream.cuda_stream if stream is not None else None)),
               "hpsgd_set_aux_stream")

    def set_recurrence(self, resident=True, spin_limit=1 << 20):
        """fp32 GRU recurrence as one launch per run of time steps (weights resident on the chip) or one per step."""
        _check(self.lib.hpsgd_set_recurrence(self._h, int(resident), int(spin_limit)), "hpsgd_set_recurrence")

    def recurrence_info(self):
        """(resident, xproj, dw): GRU layers of the last local step whose recurrence ran as resident-weight
        launches, whose forward launch did the input projection, whose backward launch accumulated dW_hh."""
        a, b, c = C.c_int(0), C.c_int(0), C.c_int(0)
        _check(self.lib.hpsgd_recurrence_info(self._h, C.byref(a), C.byref(b), C.byref(c)), "hpsgd_recurrence_info")
        return a.value, b.value, c.value

    def recurrence_gave_up(self, workspace, stream=None):
        """True if a wait inside a resident-weight recurrence launch was given up (synchronises the stream)."""
        out = C.c_int(0)
        _check(self.lib.hpsgd_recurrence_gave_up(self._h, self._ws_ptr(workspace), _stream(stream),
                                                 C.byref(out)), "hpsgd_recurrence_gave_up")
        return bool(out.value)

    # ---- kernel timing (benchmarks) ----
    def timer_enable(self, roles):
        mask = 0
        for r in roles:
            mask |= 1 << int(r)
        _check(self.lib.hpsgd_timer_enable(self._h, mask), "hpsgd_timer_enable")

    def timer_read(self, role):
        """(launch groups, total ms) of `role` since the last read; waits for the events."""
        n, ms = C.c_long(), C.c_double()
        _check(self.lib.hpsgd_timer_read(self._h, int(role), C.byref(n), C.byref(ms)), "hpsgd_timer_read")
        return int(n.value), float(ms.value)

    def role_names(self):
        return [self.lib.hpsgd_role_name(i).decode() for i in range(ROLE_COUNT)]

    def kernel_timer_enable(self, kernels):
        mask = 0
        for k in kernels:
            mask |= 1 << int(k)
        _check(self.lib.hpsgd_kernel_timer_enable(self._h, mask), "hpsgd_kernel_timer_enable")

    def kernel_timer_read(self, kernel):
        """(launches, total ms, summed algorithmic work) of `kernel` since the last read; waits for the events."""
        n, ms, w = C.c_long(), C.c_double(), C.c_double()
        _check(self.lib.hpsgd_kernel_timer_read(self._h, int(kernel), C.byref(n), C.byref(ms), C.byref(w)),
               "hpsgd_kernel_timer_read")
        return int(n.value), float(ms.value), float(w.value)

    def kernel_names(self):
        """Index = kernel id; index 0 (no kernel) is None."""
        out = [None]
        for i in range(1, KERNEL_COUNT):
            out.append(self.lib.hpsgd_kernel_name(i).decode())
        return out

    def commit_kernel_params(self):
        """Parameters per worker that went through the commit kernel in the last local step."""
        return int(self.lib.hpsgd_commit_kernel_params(self._h))

    # ---- entry points ----
    def local_step_all(self, replicas_in, replicas_out, x, y, lr, loss_out, workspace, stream=None):
        """replicas_*: float32 [K, stride] tensors (row k = worker k's flat replica)."""
        _check(self.lib.hpsgd_local_step_all(self._h, _ptr(replicas_in), _ptr(replicas_out),
                                             replicas_in.stride(0), _ptr(x), _ptr(y), float(lr),
                                             _ptr(loss_out), self._ws_ptr(workspace), _stream(stream)),
               "hpsgd_local_step_all")

    def local_step_all_cloned(self, source, replicas_out, x, y, lr, loss_out, workspace, stream=None):
        """Clone + local step as one call: parameters are read from `source` (float32 [P]), every
        worker's updated replica is written to replicas_out [K, stride]."""
        _check(self.lib.hpsgd_local_step_all_cloned(self._h, _ptr(source), _ptr(replicas_out),
                                                    replicas_out.stride(0), _ptr(x), _ptr(y), float(lr),
                                                    _ptr(loss_out), self._ws_ptr(workspace), _stream(stream)),
               "hpsgd_local_step_all_cloned")

    def local_step_all_static(self, replicas_in, replicas_out, x, y, lr, loss_out, stream=None):
        """local_step_all on the library's fixed workspace (no workspace argument, nothing allocated)."""
        _check(self.lib.hpsgd_local_step_all_static(self._h, _ptr(replicas_in), _ptr(replicas_out),
                                                    replicas_in.stride(0), _ptr(x), _ptr(y), float(lr),
                                                    _ptr(loss_out), _stream(stream)),
               "hpsgd_local_step_all_static")

    def prepare_replicas(self, replicas, workspace, stream=None):
        """Make the next local step's operand copies of the weights now (see hpsgd_prepare_replicas)."""
        _check(self.lib.hpsgd_prepare_replicas(self._h, _ptr(replicas), replicas.stride(0), self._ws_ptr(workspace),
                                               _stream(stream)), "hpsgd_prepare_replicas")

    def prepare_clones(self, global_, replicas, workspace, stream=None, with_head=False):
        """prepare_replicas for replicas that are clones of `global_`: one set of copies for all workers."""
        _check(self.lib.hpsgd_prepare_clones(self._h, _ptr(global_), _ptr(replicas), replicas.stride(0),
                                             self._ws_ptr(workspace), int(bool(with_head)), _stream(stream)),
               "hpsgd_prepare_clones")

    def local_step_all_acc(self, replicas_in, replicas_out, x, y, lr, loss_out, grad_acc, workspace, stream=None):
        """local_step_all that also adds every worker's gradient to grad_acc [K, stride]."""
        _check(self.lib.hpsgd_local_step_all_acc(self._h, _ptr(replicas_in), _ptr(replicas_out),
                                                 replicas_in.stride(0), _ptr(x), _ptr(y), float(lr),
                                                 _ptr(loss_out), _ptr(grad_acc), grad_acc.stride(0),
                                                 self._ws_ptr(workspace), _stream(stream)),
               "hpsgd_local_step_all_acc")

    def local_step(self, worker, replica_in, replica_out, x, y, lr, loss_out, workspace, stream=None):
        _check(self.lib.hpsgd_local_step(self._h, int(worker), _ptr(replica_in), _ptr(replica_out),
                                         _ptr(x), _ptr(y), float(lr), _ptr(loss_out),
                                         self._ws_ptr(workspace), _stream(stream)),
               "hpsgd_local_step")


def _ptr_array(tensors):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr()
    return arr


def merge(global_, replicas, snapshot, stream=None):
    """global += mean_k(replicas[k] - snapshot); `replicas` is a list of K flat tensors (or a [K, n] tensor)."""
    reps = list(replicas)
    P = global_.numel()
    _check(load_library().hpsgd_merge(_ptr(global_), _ptr_array(reps), _ptr(snapshot), len(reps), P,
                                      _stream(stream)), "hpsgd_merge")


def merge_sync(global_, replicas, snapshot, stream=None):
    """merge followed by sync_all of the same replicas and snapshot, in one pass."""
    reps = list(replicas)
    _check(load_library().hpsgd_merge_sync(_ptr(global_), _ptr_array(reps), _ptr(snapshot), len(reps),
                                           global_.numel(), _stream(stream)), "hpsgd_merge_sync")


def sync_replica(global_, replica, stream=None):
    _check(load_library().hpsgd_sync_replica(_ptr(global_), _ptr(replica), global_.numel(),
                                             _stream(stream)), "hpsgd_sync_replica")


def merge_snapshot(global_, replicas, snapshot, stream=None):
    """merge, then snapshot = the merged model, in one pass (the replicas are only read)."""
    reps = list(replicas)
    _check(load_library().hpsgd_merge_snapshot(_ptr(global_), _ptr_array(reps), _ptr(snapshot), len(reps),
                                               global_.numel(), _stream(stream)), "hpsgd_merge_snapshot")


def sync_all(global_, replicas, snapshot, stream=None):
    reps = list(replicas)
    _check(load_library().hpsgd_sync_all(_ptr(global_), _ptr_array(reps), len(reps), _ptr(snapshot),
                                         global_.numel(), _stream(stream)), "hpsgd_sync_all")


def gather_batch(shard, idx, n_chunks, chunk_elems, out, row_elems=None, stream=None):
    """Time-major gather: out[c, b, :] = shard[idx[b], c*chunk : (c+1)*chunk] (4-byte elements)."""
    es = shard.element_size()
    row = (shard[0].numel() if row_elems is None else row_elems) * es
    _check(load_library().hpsgd_gather_batch(_ptr(shard), _ptr(idx), idx.numel(), row, int(n_chunks),
                                             int(chunk_elems) * es, _ptr(out), _stream(stream)),
           "hpsgd_gather_batch")


def gather_batch_all(shards, idxs, n_chunks, chunk_elems, outs, row_elems=None, stream=None):
    """gather_batch for K workers in one launch (lists of K shard / index / output tensors)."""
    es = shards[0].element_size()
    row = (shards[0][0].numel() if row_elems is None else row_elems) * es
    _check(load_library().hpsgd_gather_batch_all(_ptr_array(shards), _ptr_array(idxs), len(shards),
                                                 idxs[0].numel(), row, int(n_chunks),
                                                 int(chunk_elems) * es, _ptr_array(outs), _stream(stream)),
           "hpsgd_gather_batch_all")


def probe_mfma_rate(prec, operands, iterations, result, sink, stream=None):
    """Pure-MFMA loop on every CU (argument marshalling only; see hpsgd_probe_mfma_rate).
    operands: >= 16 KiB device tensor; result: float64[4]; sink: float32[256*256]."""
    _check(load_library().hpsgd_probe_mfma_rate(PREC[prec], _ptr(operands), int(iterations), _ptr(result),
                                                _ptr(sink), _stream(stream)), "hpsgd_probe_mfma_rate")


GEMM_FORMS = {"auto": 0, "128x128": 1, "128x256": 2, "192x256": 3, "256x256": 4}


def gemm_bf16_nt(A, B, C_out, win=None, lr=0.0, form="auto", stream=None):
    """C[g] = A[g] B[g]^T, or win[g] - lr * A[g] B[g]^T (argument marshalling only; see hpsgd_gemm_bf16_nt).
    A: [G, M, Kd] and B: [G, N, Kd] torch.bfloat16, contiguous; C_out / win: [G, M, N] float32."""
    G, M, Kd = A.shape
    N = B.shape[1]
    assert B.shape == (G, N, Kd) and C_out.shape == (G, M, N) and A.is_contiguous() and B.is_contiguous()
    assert C_out.is_contiguous() and (win is None or (win.shape == C_out.shape and win.is_contiguous()))
    _check(load_library().hpsgd_gemm_bf16_nt(_ptr(A), Kd, M * Kd, _ptr(B), Kd, N * Kd, _ptr(C_out), N, M * N,
                                             _ptr(win) if win is not None else None, M * N, float(lr), M, N, Kd, G,
                                             GEMM_FORMS[form], _stream(stream)), "hpsgd_gemm_bf16_nt")


def delay_us(microseconds, stream=None):
    """Occupy `stream` for about that long (synthetic synchronisation latency)."""
    _check(load_library().hpsgd_delay_us(int(microseconds), _stream(stream)), "hpsgd_delay_us")


def merge_grad(global_, grad_accs, lr, stream=None):
    """global -= lr * mean_k grad_accs[k] (Eq. 1 as printed)."""
    _check(load_library().hpsgd_merge_grad(_ptr(global_), _ptr_array(grad_accs), float(lr), len(grad_accs),
                                           global_.numel(), _stream(stream)), "hpsgd_merge_grad")
