"""Pins for the oracle's model arithmetic (forward, BPTT, MLP backward, loss).

None of these re-types the oracle's formulas: they use central finite differences
of the oracle's own loss, a double-precision library GRU with autograd (the cell of
the library the paper ran on, Sec. 4.1 "Softwares"), and closed forms.
"""
import math

import numpy as np
import pytest
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

from oracle import hpsgd_oracle as oc
from paper_2009_02701_amd import workloads as wl


def _batch(cfg, worker=0, step=0):
    x, y = wl.make_shard(cfg, worker)
    return oc.gather_batch(cfg["kind"], x, y, wl.batch_indices(cfg, worker, step))


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


# ---------------------------------------------------------------------------- batch gather
def test_gather_batch_hand_written_examples():
    """Sec. 3.2: a worker's mini-batch out of its sub-dataset.  The expected arrays are typed out
    by hand (not produced by indexing code): a wrong axis order, a missing shift of the targets
    or an off-by-one in the sample number changes them."""
    # classifier: 4 samples of T = 2 steps x I = 3 features; sample n, step t, feature i = 100n + 10t + i
    samples = np.array([[[0, 1, 2], [10, 11, 12]],
                        [[100, 101, 102], [110, 111, 112]],
                        [[200, 201, 202], [210, 211, 212]],
                        [[300, 301, 302], [310, 311, 312]]], np.float32)
    labels = np.array([7, 5, 3, 1], np.int32)
    x, y = oc.gather_batch("gru_cls", samples, labels, np.array([2, 0, 3], np.int32))
    want_x = np.array([[[200, 201, 202], [0, 1, 2], [300, 301, 302]],          # step 0 of samples 2, 0, 3
                       [[210, 211, 212], [10, 11, 12], [310, 311, 312]]],       # step 1
                      np.float32)
    assert x.dtype == np.float32 and x.shape == (2, 3, 3) and np.array_equal(x, want_x)
    assert y.dtype == np.int32 and np.array_equal(y, np.array([3, 7, 1], np.int32))
    # MLP: rows as they are
    flat = np.array([[1, 2], [3, 4], [5, 6]], np.float32)
    x, y = oc.gather_batch("mlp", flat, np.array([9, 8, 7], np.int32), np.array([1, 1, 2], np.int32))
    assert np.array_equal(x, np.array([[3, 4], [3, 4], [5, 6]], np.float32))
    assert np.array_equal(y, np.array([8, 8, 7], np.int32))
    # language model: samples are runs of T + 1 = 4 tokens; inputs = first 3, targets = last 3
    tok = np.array([[11, 12, 13, 14],
                    [21, 22, 23, 24],
                    [31, 32, 33, 34]], np.int32)
    x, y = oc.gather_batch("gru_lm", tok, None, np.array([2, 0], np.int32))
    assert np.array_equal(x, np.array([[31, 11], [32, 12], [33, 13]], np.int32))
    assert np.array_equal(y, np.array([[32, 12], [33, 13], [34, 14]], np.int32))


def test_gather_batch_is_a_selection_of_the_shard():
    """Every gathered value is the shard's value at the named sample, for a seeded shard and the
    seeded batch order; the targets of the language model are its inputs one token later."""
    for name in ("tiny_gru", "mlp", "gru_lm"):
        cfg = wl.scaled(wl.CONFIGS[name], batch=6) if name != "gru_lm" else wl.scaled(
            wl.CONFIGS[name], batch=6, seq_len=9, vocab=50)
        if name == "mlp":
            cfg = wl.scaled(cfg, dims=[12, 8, 4])
        xs, ys = wl.make_shard(cfg, 1)
        idx = wl.batch_indices(cfg, 1, 5)
        x, y = oc.gather_batch(cfg["kind"], xs, ys, idx)
        rng = np.random.default_rng(3)
        for _ in range(50):
            b = int(rng.integers(0, len(idx)))
            if cfg["kind"] == "gru_cls":
                t, i = int(rng.integers(0, cfg["seq_len"])), int(rng.integers(0, cfg["input"]))
                assert x[t, b, i] == xs[idx[b], t, i] and y[b] == ys[idx[b]]
            elif cfg["kind"] == "mlp":
                i = int(rng.integers(0, cfg["dims"][0]))
                assert x[b, i] == xs[idx[b], i] and y[b] == ys[idx[b]]
            else:
                t = int(rng.integers(0, cfg["seq_len"]))
                assert x[t, b] == xs[idx[b], t] and y[t, b] == xs[idx[b], t + 1]
                if t + 1 < cfg["seq_len"]:
                    assert y[t, b] == x[t + 1, b]


# ---------------------------------------------------------------------------- rounded-operand mode
def test_round_bf16_matches_the_library_conversion_and_hand_written_ties():
    """tests/parity.py::round_bf16 (nearest, ties to even, 8 significand bits) against the
    library's float32 -> bfloat16 conversion on random values of many magnitudes, and on ties
    written out by hand."""
    from parity import round_bf16
    rng = np.random.default_rng(11)
    v = (rng.standard_normal(200_000) * np.exp(rng.uniform(-30, 30, 200_000))).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(round_bf16(v), want)
    # bf16 has 7 stored fraction bits: the spacing at 1.0 is 2^-7
    ulp = 2.0 ** -7
    cases = {
        1.0: 1.0,
        1.0 + ulp / 2: 1.0,                 # tie -> even (fraction 0)
        1.0 + ulp + ulp / 2: 1.0 + 2 * ulp,  # tie -> even (fraction 2)
        1.0 + ulp / 2 + 2.0 ** -20: 1.0 + ulp,  # just above the tie
        1.0 + ulp / 2 - 2.0 ** -20: 1.0,        # just below
        -(1.0 + ulp + ulp / 2): -(1.0 + 2 * ulp),
        0.0: 0.0,
        3.0e38: float(np.float32(2.0 ** 127 * (1 + 98 / 128))),  # nearest bf16 of 3e38
    }
    for x, r in cases.items():
        assert float(round_bf16(np.float32(x)).reshape(-1)[0]) == r, (x, r)


class _RoundedMM(torch.autograd.Function):
    """a @ b with both operands rounded to bf16, in the forward product and in both products of
    the backward pass (upstream gradient and the other factor): the rule of the bf16 path."""

    @staticmethod
    def r(t):
        return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    @staticmethod
    def forward(ctx, a, b):
        ctx.save_for_backward(a, b)
        return _RoundedMM.r(a) @ _RoundedMM.r(b)

    @staticmethod
    def backward(ctx, g):
        a, b = ctx.saved_tensors
        r = _RoundedMM.r
        return r(g) @ r(b).T, r(a).T @ r(g)


def _torch_rounded_loss_and_grads(params, x, y):
    """The model in double precision with the library's autograd for everything that is not a
    matrix product; every matrix product through _RoundedMM."""
    p = {k: torch.tensor(np.asarray(v, np.float64), requires_grad=True) for k, v in params.items()}
    mm = _RoundedMM.apply
    if "fc0.W" in p:
        a = torch.tensor(np.asarray(x, np.float64))
        L = sum(1 for k in p if k.endswith(".W"))
        for i in range(L):
            a = mm(a, p[f"fc{i}.W"].T) + p[f"fc{i}.b"]
            if i < L - 1:
                a = torch.relu(a)
        logits, tgt = a, torch.tensor(np.asarray(y), dtype=torch.long)
    else:
        lm = "embed.E" in p
        inp = p["embed.E"][torch.tensor(np.asarray(x), dtype=torch.long)] if lm else torch.tensor(np.asarray(x, np.float64))
        T, B = inp.shape[0], inp.shape[1]
        L = sum(1 for k in p if k.endswith(".W_hh"))
        for l in range(L):
            W_ih, W_hh, b_ih, b_hh = (p[f"l{l}.{n}"] for n in ("W_ih", "W_hh", "b_ih", "b_hh"))
            H = W_hh.shape[1]
            h = torch.zeros(B, H, dtype=torch.float64)
            outs = []
            for t in range(T):
                gx = mm(inp[t], W_ih.T) + b_ih
                gh = mm(h, W_hh.T) + b_hh
                r = torch.sigmoid(gx[:, :H] + gh[:, :H])
                z = torch.sigmoid(gx[:, H:2 * H] + gh[:, H:2 * H])
                n = torch.tanh(gx[:, 2 * H:] + r * gh[:, 2 * H:])
                h = (1 - z) * n + z * h
                outs.append(h)
            inp = torch.stack(outs)
        if lm:
            logits = mm(inp.reshape(T * B, -1), p["head.W"].T) + p["head.b"]
            tgt = torch.tensor(np.asarray(y).reshape(-1), dtype=torch.long)
        else:
            logits = mm(inp[-1], p["head.W"].T) + p["head.b"]
            tgt = torch.tensor(np.asarray(y), dtype=torch.long)
    loss = torch.nn.functional.cross_entropy(logits, tgt)
    loss.backward()
    return float(loss), {k: (v.grad.numpy() if v.grad is not None else np.zeros(v.shape)) for k, v in p.items()}


@pytest.mark.parametrize("name", ["lm", "cls2", "mlp"])
def test_rounded_operand_mode_rounds_exactly_the_matrix_products(name):
    """The oracle's rnd= mode (used for the tight bar of the bf16 parity tests) against the
    library's autograd with every matrix product - and nothing else - taking bf16-rounded
    operands.  A product the oracle forgot to round, or a rounding applied to something that is
    not a GEMM operand (a bias sum, the embedding gradient), shows as an error of the order of
    the bf16 spacing (4e-3); agreement is at float64 rounding."""
    from parity import round_bf16
    cfg = {"lm": wl.scaled(wl.CONFIGS["gru_lm"], vocab=40, embed=12, hidden=16, seq_len=5, batch=6, K=1),
           "cls2": wl.scaled(wl.CONFIGS["gru_cls"], layers=2, input=10, hidden=16, seq_len=4, batch=5, K=1),
           "mlp": wl.scaled(wl.CONFIGS["mlp"], dims=[20, 24, 16, 5], batch=9, K=1)}[name]
    params = wl.init_params(cfg)
    x, y = _batch(cfg)
    loss, g = oc.loss_and_grads(params, x, y, rnd=round_bf16)
    tl, tg = _torch_rounded_loss_and_grads(params, x, y)
    assert abs(loss - tl) <= 1e-12 * abs(tl)
    for k in g:
        scale = max(np.abs(tg[k]).max(), 1e-30)
        assert np.abs(g[k] - tg[k]).max() <= 1e-11 * scale, k
    # and the mode does change the result (it is not a no-op)
    l0, g0 = oc.loss_and_grads(params, x, y)
    assert abs(l0 - loss) > 1e-7


def test_mlp_relu_branch_hook_is_the_derivative_through_the_other_branch():
    """mlp_loss_and_grads(flip=...): for the named hidden units the backward pass takes the other
    branch of the ReLU.  Pinned with the library's autograd on a network whose ReLU derivative is
    an explicit constant mask (the forward values stay those of the ReLU); with no unit named the
    gradients are the plain ones."""
    cfg = wl.scaled(wl.CONFIGS["mlp"], dims=[20, 24, 16, 5], batch=9, K=1)
    params = wl.init_params(cfg)
    x, y = _batch(cfg)
    pre = oc.mlp_preactivations(params, x)
    assert [a.shape for a in pre] == [(9, 24), (9, 16)]
    flips = [(0, 1, 2), (0, 3, 7), (1, 8, 15), (1, 0, 0)]
    masks = [a > 0.0 for a in pre]
    for (i, b, j) in flips:
        masks[i][b, j] = not masks[i][b, j]
    p = {k: torch.tensor(np.asarray(v, np.float64), requires_grad=True) for k, v in params.items()}
    h = torch.tensor(np.asarray(x, np.float64))
    for i in range(3):
        a = h @ p[f"fc{i}.W"].T + p[f"fc{i}.b"]
        if i < 2:
            m = torch.tensor(masks[i].astype(np.float64))
            h = a * m + (torch.relu(a) - a * m).detach()
        else:
            h = a
    loss = torch.nn.functional.cross_entropy(h, torch.tensor(np.asarray(y), dtype=torch.long))
    loss.backward()
    l, g = oc.mlp_loss_and_grads(params, x, y, flip=flips)
    assert abs(l - float(loss)) <= 1e-12
    for k in g:
        assert np.abs(g[k] - p[k].grad.numpy()).max() <= 1e-12 * max(1.0, np.abs(g[k]).max()), k
    l0, g0 = oc.mlp_loss_and_grads(params, x, y)
    l1, g1 = oc.mlp_loss_and_grads(params, x, y, flip=())
    assert l0 == l1 and all(np.array_equal(g0[k], g1[k]) for k in g0)
    assert np.abs(g0["fc0.W"] - g["fc0.W"]).max() > 1e-6
