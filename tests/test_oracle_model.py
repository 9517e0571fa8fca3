"""Pins for the oracle's model arithmetic (forward, BPTT, MLP backward, loss).

None of these re-types the oracle's formulas: they use central finite differences
of the oracle's own loss, a double-precision library GRU with autograd (the cell of
the library the paper ran on, Sec. 4.1 "Softwares"), and closed forms.
"""
import math

import numpy as np
import pytest
import torch

from oracle import hpsgd_oracle as oc
from paper_2009_02701_amd import workloads as wl


def _batch(cfg, worker=0, step=0):
    return wl.host_batch(cfg, wl.make_shard(cfg, worker), wl.batch_indices(cfg, worker, step))


def _fd_check(params, x, y, names=None, eps=1e-6, tol=1e-6, stride=1):
    """Central differences on (a strided subset of) every parameter tensor."""
    p64 = {k: np.asarray(v, np.float64).copy() for k, v in params.items()}
    _, g = oc.loss_and_grads(p64, x, y)
    for name in (names or list(p64)):
        flat = p64[name].reshape(-1)
        fd = np.zeros(flat.size)
        idx = np.arange(0, flat.size, stride)
        for j in idx:
            keep = flat[j]
            flat[j] = keep + eps
            lp = oc.loss_and_grads(p64, x, y)[0]
            flat[j] = keep - eps
            lm = oc.loss_and_grads(p64, x, y)[0]
            flat[j] = keep
            fd[j] = (lp - lm) / (2 * eps)
        an = g[name].reshape(-1)[idx]
        scale = max(np.abs(an).max(), 1e-12)
        err = np.abs(fd[idx] - an).max() / scale
        assert err < tol, (name, err)


def test_fd_tiny_gru_every_parameter():
    """Config 1 shapes, all 5130 parameters."""
    cfg = wl.CONFIGS["tiny_gru"]
    assert wl.param_count(cfg) == 5130
    x, y = _batch(cfg)
    _fd_check(wl.init_params(cfg), x, y)


def test_fd_two_layer_lm():
    cfg = wl.scaled(wl.CONFIGS["gru_lm"], vocab=11, embed=5, hidden=6, seq_len=4, batch=3)
    x, y = _batch(cfg)
    # make sure a token id repeats inside the batch (duplicate rows must be summed)
    assert len(np.unique(x)) < x.size
    _fd_check(wl.init_params(cfg), x, y)


def test_fd_mlp():
    cfg = wl.scaled(wl.CONFIGS["mlp"], dims=[7, 9, 8, 4], batch=5)
    x, y = _batch(cfg)
    _fd_check(wl.init_params(cfg), x, y)


def _torch_gru_reference(cfg, params, x, y):
    """The same model built from torch.nn modules in double, gradients by autograd."""
    lm = cfg["kind"] == "gru_lm"
    H, L = cfg["hidden"], cfg["layers"]
    width = cfg["embed"] if lm else cfg["input"]
    gru = torch.nn.GRU(width, H, num_layers=L).double()
    classes = cfg["vocab"] if lm else cfg["classes"]
    head = torch.nn.Linear(H, classes).double()
    emb = torch.nn.Embedding(cfg["vocab"], cfg["embed"]).double() if lm else None
    t = lambda a: torch.tensor(np.asarray(a, np.float64))
    with torch.no_grad():
        for l in range(L):
            getattr(gru, f"weight_ih_l{l}").copy_(t(params[f"l{l}.W_ih"]))
            getattr(gru, f"weight_hh_l{l}").copy_(t(params[f"l{l}.W_hh"]))
            getattr(gru, f"bias_ih_l{l}").copy_(t(params[f"l{l}.b_ih"]))
            getattr(gru, f"bias_hh_l{l}").copy_(t(params[f"l{l}.b_hh"]))
        head.weight.copy_(t(params["head.W"]))
        head.bias.copy_(t(params["head.b"]))
        if lm:
            emb.weight.copy_(t(params["embed.E"]))
    if lm:
        inp = emb(torch.tensor(np.asarray(x, np.int64)))
        out, _ = gru(inp)
        logits = head(out.reshape(-1, H))
        loss = torch.nn.functional.cross_entropy(logits, torch.tensor(np.asarray(y, np.int64)).reshape(-1))
    else:
        out, _ = gru(t(x))
        logits = head(out[-1])
        loss = torch.nn.functional.cross_entropy(logits, torch.tensor(np.asarray(y, np.int64)))
    loss.backward()
    g = {}
    for l in range(L):
        g[f"l{l}.W_ih"] = getattr(gru, f"weight_ih_l{l}").grad.numpy()
        g[f"l{l}.W_hh"] = getattr(gru, f"weight_hh_l{l}").grad.numpy()
        g[f"l{l}.b_ih"] = getattr(gru, f"bias_ih_l{l}").grad.numpy()
        g[f"l{l}.b_hh"] = getattr(gru, f"bias_hh_l{l}").grad.numpy()
    g["head.W"], g["head.b"] = head.weight.grad.numpy(), head.bias.grad.numpy()
    if lm:
        g["embed.E"] = emb.weight.grad.numpy()
    return float(loss), g


@pytest.mark.parametrize("case", ["tiny_gru", "cls_2layer", "lm_2layer"])
def test_against_library_gru_double(case):
    if case == "tiny_gru":
        cfg = wl.CONFIGS["tiny_gru"]
    elif case == "cls_2layer":
        cfg = wl.scaled(wl.CONFIGS["gru_cls"], layers=2, input=12, hidden=20, seq_len=9, batch=6)
    else:
        cfg = wl.scaled(wl.CONFIGS["gru_lm"], vocab=50, embed=12, hidden=24, seq_len=7, batch=5)
    params = wl.init_params(cfg)
    x, y = _batch(cfg)
    loss, g = oc.loss_and_grads(params, x, y)
    rloss, rg = _torch_gru_reference(cfg, params, x, y)
    assert abs(loss - rloss) < 1e-12 * max(1, abs(rloss))
    assert set(g) == set(rg)
    for k in g:
        assert g[k].shape == rg[k].shape
        assert np.abs(g[k] - rg[k]).max() <= 1e-11 * max(np.abs(rg[k]).max(), 1e-30), k


def test_against_library_mlp_double():
    cfg = wl.scaled(wl.CONFIGS["mlp"], dims=[20, 16, 12, 10], batch=8)
    params = wl.init_params(cfg)
    x, y = _batch(cfg)
    loss, g = oc.loss_and_grads(params, x, y)
    ws = [torch.tensor(np.asarray(params[f"fc{i}.W"], np.float64), requires_grad=True) for i in range(3)]
    bs = [torch.tensor(np.asarray(params[f"fc{i}.b"], np.float64), requires_grad=True) for i in range(3)]
    a = torch.tensor(np.asarray(x, np.float64))
    for i in range(3):
        a = torch.nn.functional.linear(a, ws[i], bs[i])
        if i < 2:
            a = torch.relu(a)
    rl = torch.nn.functional.cross_entropy(a, torch.tensor(np.asarray(y, np.int64)))
    rl.backward()
    assert abs(loss - float(rl)) < 1e-12
    for i in range(3):
        assert np.abs(g[f"fc{i}.W"] - ws[i].grad.numpy()).max() < 1e-12
        assert np.abs(g[f"fc{i}.b"] - bs[i].grad.numpy()).max() < 1e-12


def test_zero_weights_loss_is_ln_classes():
    """All-zero parameters give uniform class probabilities: loss = ln C exactly."""
    for name in ("tiny_gru", "mlp"):
        cfg = wl.CONFIGS[name] if name == "tiny_gru" else wl.scaled(wl.CONFIGS["mlp"], dims=[6, 5, 10], batch=4)
        params = {k: np.zeros_like(v) for k, v in wl.init_params(cfg).items()}
        x, y = _batch(cfg)
        loss, g = oc.loss_and_grads(params, x, y)
        assert abs(loss - math.log(10.0)) < 1e-14
    lm = wl.scaled(wl.CONFIGS["gru_lm"], vocab=17, embed=4, hidden=5, seq_len=3, batch=2)
    params = {k: np.zeros_like(v) for k, v in wl.init_params(lm).items()}
    loss, _ = oc.loss_and_grads(params, *_batch(lm))
    assert abs(loss - math.log(17.0)) < 1e-14


def test_single_step_closed_form():
    """T = 1 with h_0 = 0: q = b_hn, so h_1 = (1 - z) * tanh(a_n), written out per unit by hand."""
    cfg = wl.scaled(wl.CONFIGS["tiny_gru"], seq_len=1, input=3, hidden=2, batch=2)
    p = {k: np.asarray(v, np.float64) for k, v in wl.init_params(cfg).items()}
    x, _ = _batch(cfg)
    hs, _ = oc.gru_layer_forward(p["l0.W_ih"], p["l0.W_hh"], p["l0.b_ih"], p["l0.b_hh"],
                                 np.asarray(x, np.float64))
    H = 2
    for b in range(2):
        for j in range(H):
            pre = lambda g: sum(p["l0.W_ih"][g * H + j, i] * float(x[0, b, i]) for i in range(3)) \
                + p["l0.b_ih"][g * H + j]
            r = 1 / (1 + math.exp(-(pre(0) + p["l0.b_hh"][j])))
            z = 1 / (1 + math.exp(-(pre(1) + p["l0.b_hh"][H + j])))
            n = math.tanh(pre(2) + r * p["l0.b_hh"][2 * H + j])
            assert abs(hs[1, b, j] - (1 - z) * n) < 1e-15
    assert np.all(hs[0] == 0)


def test_softmax_ce_bruteforce():
    g = np.random.default_rng(5)
    logits = g.standard_normal((6, 7)) * 3
    y = g.integers(0, 7, 6)
    loss, d = oc.softmax_ce(logits, y)
    tot = 0.0
    for i in range(6):
        den = sum(math.exp(v) for v in logits[i])
        tot += -math.log(math.exp(logits[i, y[i]]) / den)
        for c in range(7):
            want = (math.exp(logits[i, c]) / den - (1.0 if c == y[i] else 0.0)) / 6
            assert abs(d[i, c] - want) < 1e-14
    assert abs(loss - tot / 6) < 1e-13
    # shift invariance / large logits do not overflow
    loss2, _ = oc.softmax_ce(logits + 1000.0, y)
    assert abs(loss2 - loss) < 1e-9
