"""Seeded synthetic workloads: the five configurations and their input generators.

This module holds NO arithmetic of the method (no forward pass, no gradient, no
update rule).  It only names the workloads and draws their inputs, so that the
CPU oracle tests and the HIP path can be fed the very same numbers.  It imports
numpy only; it never imports the HIP binding nor the oracle.

The paper trains CNNs on an image dataset with per-worker batch 128, lr 0.01 and
4..16 workers (Sec. 4.1); those models and that dataset are replaced here by
synthetic GRU / MLP workloads of the same structure (per-worker batch, worker
counts, a GRU as the high communication-to-computation model of Sec. 1).

Every random stream is `numpy.random.Philox` keyed by
(BASE_SEED, config id, tensor id, worker, step): values are drawn in float64,
rounded once to float32, and both sides start from those float32 numbers.
"""
from __future__ import annotations

import math
import zlib

import numpy as np

BASE_SEED = 200902701
SHARD_BATCHES = 8  # every worker's sub-dataset holds 8 mini-batches

CONFIGS = {
    # Tiny GRU classifier (oracle finishes in milliseconds)
    "tiny_gru": dict(id=1, kind="gru_cls", prec="fp32", layers=1, input=16, hidden=32,
                     seq_len=8, batch=4, classes=10, K=2, lr=0.1),
    # GRU classifier: the configuration the headline metric is quoted on
    "gru_cls": dict(id=2, kind="gru_cls", prec="fp32", layers=1, input=128, hidden=512,
                    seq_len=35, batch=64, classes=10, K=4, lr=0.05),
    # GRU language model, bf16 GEMM operands / fp32 accumulate / fp32 master params
    "gru_lm": dict(id=3, kind="gru_lm", prec="bf16", layers=2, vocab=10000, embed=256,
                   hidden=1024, seq_len=35, batch=32, K=8, lr=0.05),
    # MLP, merge-heavy (low compute-to-parameter ratio)
    "mlp": dict(id=4, kind="mlp", prec="fp32", dims=[784, 1024, 1024, 10], batch=128,
                K=16, lr=0.01),
    # merge-only stress: flat parameter vector
    "merge_stress": dict(id=5, kind="flat", P=100_000_000, K=8, iters=50),
}


def scaled(cfg: dict, **over) -> dict:
    """A copy of a configuration with some sizes overridden (test cases)."""
    out = dict(cfg)
    out.update(over)
    return out


def _rng(cfg: dict, tensor: str, worker: int = 0, step: int = 0) -> np.random.Generator:
    tid = zlib.crc32(tensor.encode()) & 0xFFFFFFFF
    key1 = ((cfg["id"] & 0xFF) << 56) | (tid << 24) | ((worker & 0xFFF) << 12) | (step & 0xFFF)
    return np.random.Generator(np.random.Philox(key=[BASE_SEED, key1]))


# ----------------------------------------------------------------------------
# parameter tensors: names, shapes, init distributions
# ----------------------------------------------------------------------------
def param_shapes(cfg: dict) -> list[tuple[str, tuple[int, ...]]]:
    """Ordered (name, shape) list of a model's parameter tensors.

    Matrices are [out, in] row-major; a GRU layer stacks its three gates in the
    order r, z, n along `out` and carries two bias vectors.
    """
    kind = cfg["kind"]
    out: list[tuple[str, tuple[int, ...]]] = []
    if kind in ("gru_cls", "gru_lm"):
        H = cfg["hidden"]
        if kind == "gru_lm":
            out.append(("embed.E", (cfg["vocab"], cfg["embed"])))
            width, classes = cfg["embed"], cfg["vocab"]
        else:
            width, classes = cfg["input"], cfg["classes"]
        for l in range(cfg["layers"]):
            out.append((f"l{l}.W_ih", (3 * H, width)))
            out.append((f"l{l}.W_hh", (3 * H, H)))
            out.append((f"l{l}.b_ih", (3 * H,)))
            out.append((f"l{l}.b_hh", (3 * H,)))
            width = H
        out.append(("head.W", (classes, H)))
        out.append(("head.b", (classes,)))
    elif kind == "mlp":
        d = cfg["dims"]
        for i in range(len(d) - 1):
            out.append((f"fc{i}.W", (d[i + 1], d[i])))
            out.append((f"fc{i}.b", (d[i + 1],)))
    else:
        raise ValueError(kind)
    return out


def param_count(cfg: dict) -> int:
    return sum(int(np.prod(s)) for _, s in param_shapes(cfg))


def init_params(cfg: dict) -> dict[str, np.ndarray]:
    """Initial global model as float32 tensors keyed by name.

    GRU and head: U(-1/sqrt(H), 1/sqrt(H)); embedding: N(0,1);
    MLP: weights U(+-sqrt(6/fan_in)), biases U(+-1/sqrt(fan_in)).
    """
    out = {}
    for name, shape in param_shapes(cfg):
        g = _rng(cfg, "param:" + name)
        if cfg["kind"] == "mlp":
            layer = int(name[2:name.index(".")])
            fan_in = cfg["dims"][layer]
            bound = math.sqrt(6.0 / fan_in) if name.endswith(".W") else 1.0 / math.sqrt(fan_in)
            v = g.uniform(-bound, bound, size=shape)
        elif name == "embed.E":
            v = g.standard_normal(size=shape)
        else:
            bound = 1.0 / math.sqrt(cfg["hidden"])
            v = g.uniform(-bound, bound, size=shape)
        out[name] = v.astype(np.float32)
    return out


# ----------------------------------------------------------------------------
# data shards (each worker's sub-dataset) and batch selection
# ----------------------------------------------------------------------------
def zipf_ids(g: np.random.Generator, vocab: int, size, s: float = 1.1) -> np.ndarray:
    """Bounded Zipf token ids: id = rank-1, P(rank) ~ rank**-s, rank in 1..vocab."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = g.random(size=size)
    ids = np.searchsorted(cdf, u, side="right")
    return np.minimum(ids, vocab - 1).astype(np.int32)


def make_shard(cfg: dict, worker: int) -> tuple[np.ndarray, np.ndarray | None]:
    """Worker's sub-dataset: (samples, labels).

    gru_cls: x float32 [N, T, I], y int32 [N];  mlp: x float32 [N, D0], y int32 [N];
    gru_lm: tokens int32 [N, T+1], labels None (targets are the shifted tokens).
    N = SHARD_BATCHES * batch.
    """
    n = SHARD_BATCHES * cfg["batch"]
    kind = cfg["kind"]
    gx = _rng(cfg, "shard:x", worker)
    gy = _rng(cfg, "shard:y", worker)
    if kind == "gru_cls":
        x = gx.standard_normal(size=(n, cfg["seq_len"], cfg["input"])).astype(np.float32)
        y = gy.integers(0, cfg["classes"], size=n).astype(np.int32)
        return x, y
    if kind == "mlp":
        x = gx.random(size=(n, cfg["dims"][0])).astype(np.float32)
        y = gy.integers(0, cfg["dims"][-1], size=n).astype(np.int32)
        return x, y
    if kind == "gru_lm":
        return zipf_ids(gx, cfg["vocab"], (n, cfg["seq_len"] + 1)), None
    raise ValueError(kind)


def batch_order(cfg: dict, worker: int) -> np.ndarray:
    """Seeded permutation of the worker's shard; step s takes the s-th B-slice (mod 8)."""
    n = SHARD_BATCHES * cfg["batch"]
    return _rng(cfg, "shard:perm", worker).permutation(n).astype(np.int32)


def batch_indices(cfg: dict, worker: int, step: int) -> np.ndarray:
    b = cfg["batch"]
    s = step % SHARD_BATCHES
    return batch_order(cfg, worker)[s * b:(s + 1) * b].copy()


# ----------------------------------------------------------------------------
# merge-only stress (flat vectors)
# ----------------------------------------------------------------------------
def flat_base(cfg: dict, P: int | None = None) -> np.ndarray:
    """Base flat vector U(-1, 1), float32."""
    P = cfg["P"] if P is None else P
    return _rng(cfg, "flat:base").uniform(-1.0, 1.0, size=P).astype(np.float32)


def flat_delta(cfg: dict, worker: int, P: int | None = None) -> np.ndarray:
    """Worker's replica displacement N(0, (1e-3)^2), float32."""
    P = cfg["P"] if P is None else P
    return (1e-3 * _rng(cfg, "flat:delta", worker).standard_normal(size=P)).astype(np.float32)
