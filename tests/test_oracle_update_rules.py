"""Pins for the oracle's commit, merge, sync and schedules (Alg. 1-3, Eq. 1-2, Sec. 3.2)."""
import cmath

import numpy as np

from oracle import hpsgd_oracle as oc
from paper_2009_02701_amd import workloads as wl

CFG = wl.CONFIGS["tiny_gru"]


def _batch_fn(cfg):
    shards = [wl.make_shard(cfg, k) for k in range(cfg["K"])]
    return lambda k, s: oc.gather_batch(cfg["kind"], shards[k][0], shards[k][1], wl.batch_indices(cfg, k, s))


def _close(a, b, tol=1e-12):
    for k in a:
        assert np.abs(np.asarray(a[k]) - np.asarray(b[k])).max() <= tol * max(1.0, np.abs(b[k]).max()), k


# ----------------------------------------------------------------------------- merge (Eq. 1 / Eq. 2)
def test_merge_bruteforce_loops():
    g = np.random.default_rng(1)
    P, K = 13, 3
    G, S = g.standard_normal(P), g.standard_normal(P)
    R = [g.standard_normal(P) for _ in range(K)]
    out = oc.merge(G, R, S)
    for j in range(P):
        acc = 0.0
        for k in range(K):
            acc += R[k][j] - S[j]
        assert abs(out[j] - (G[j] + acc / K)) < 1e-15


def test_merge_equals_replica_average_eq2():
    """Eq. 2: committing the averaged accumulated gradients to the previous global model
    gives the plain average of the workers' models (global == snapshot)."""
    g = np.random.default_rng(2)
    S = g.standard_normal(100)
    R = [S + 1e-2 * g.standard_normal(100) for _ in range(5)]
    out = oc.merge(S.copy(), R, S)
    assert np.abs(out - np.mean(R, axis=0)).max() < 1e-15


def test_merge_identical_replicas_and_single_worker():
    g = np.random.default_rng(3)
    G, S = g.standard_normal(50), g.standard_normal(50)
    r = S + g.standard_normal(50)
    assert np.abs(oc.merge(G, [r] * 4, S) - (G + (r - S))).max() < 1e-15
    assert np.abs(oc.merge(G, [r], S) - (G + (r - S))).max() == 0.0


def test_merge_is_eq1_with_accumulated_gradients():
    """Eq. 1 literally: W_prev - mu * sum_i sum_e grad_i^e / n, with the gradients
    accumulated while the replicas were being trained."""
    bf = _batch_fn(CFG)
    init = {k: v.astype(np.float64) for k, v in wl.init_params(CFG).items()}
    K, lr, steps = CFG["K"], CFG["lr"], 3
    acc = [{k: np.zeros_like(v) for k, v in init.items()} for _ in range(K)]
    R = [oc.sync(init) for _ in range(K)]
    for e in range(steps):
        for i in range(K):
            _, grads = oc.loss_and_grads(R[i], *bf(i, e))
            for k in grads:
                acc[i][k] += grads[k]
            R[i], _ = oc.local_step(R[i], *bf(i, e), lr)
    want = {k: init[k] - lr * sum(acc[i][k] for i in range(K)) / K for k in init}
    _close(oc.merge(init, R, init), want)


# ----------------------------------------------------------------------------- commit / sync
def test_commit_lr_zero_and_linearity():
    p = wl.init_params(CFG)
    x, y = _batch_fn(CFG)(0, 0)
    new, _ = oc.local_step(p, x, y, 0.0)
    for k in p:
        assert np.array_equal(new[k], p[k].astype(np.float64))
    a, _ = oc.local_step(p, x, y, 0.1)
    b, _ = oc.local_step(p, x, y, 0.2)
    for k in p:
        assert np.abs((b[k] - p[k]) - 2 * (a[k] - p[k])).max() < 1e-15


def test_sync_is_exact_copy():
    p = wl.init_params(CFG)
    c = oc.sync(p)
    for k in p:
        assert c[k] is not p[k] and np.array_equal(c[k], p[k]) and c[k].dtype == p[k].dtype


# ----------------------------------------------------------------------------- schedules
def test_sseq_gamma1_is_ssgd_on_the_concatenated_batch():
    """One local step per round == SGD with the average of the workers' gradients
    == one SGD step on the K*B batch with mean loss (SSGD, Sec. 2)."""
    bf = _batch_fn(CFG)
    init = wl.init_params(CFG)
    K, lr = CFG["K"], CFG["lr"]
    G, _ = oc.s_seq(init, bf, K, lr, gamma=1, rounds=3)
    W = {k: v.astype(np.float64) for k, v in init.items()}
    for s in range(3):
        xs, ys = zip(*[bf(k, s) for k in range(K)])
        x = np.concatenate(xs, axis=1)          # time-major: batch is axis 1
        y = np.concatenate(ys, axis=0)
        _, g = oc.loss_and_grads(W, x, y)
        W = {k: W[k] - lr * g[k] for k in W}
    _close(G, W)


def test_sseq_is_local_sgd_model_averaging():
    """Alg. 1: gamma local updates per worker, then the models are averaged."""
    bf = _batch_fn(CFG)
    init = wl.init_params(CFG)
    K, lr, gamma, rounds = CFG["K"], CFG["lr"], 3, 2
    G, _ = oc.s_seq(init, bf, K, lr, gamma=gamma, rounds=rounds)
    w = [{k: v.astype(np.float64) for k, v in init.items()} for _ in range(K)]
    e = 0
    for _ in range(rounds):
        for _ in range(gamma):
            for i in range(K):
                _, g = oc.loss_and_grads(w[i], *bf(i, e))
                w[i] = {k: w[i][k] - lr * g[k] for k in g}
            e += 1
        avg = {k: sum(w[i][k] for i in range(K)) / K for k in init}
        w = [dict(avg) for _ in range(K)]
    _close(G, w[0])


def test_sseq_single_worker_is_plain_sgd():
    bf = _batch_fn(CFG)
    init = wl.init_params(CFG)
    G, _ = oc.s_seq(init, bf, 1, 0.1, gamma=2, rounds=2)
    W = {k: v.astype(np.float64) for k, v in init.items()}
    for s in range(4):
        W, _ = oc.local_step(W, *bf(0, s), 0.1)
    _close(G, W)


def test_psgd_is_plain_sgd_per_worker_and_averages_to_one_long_local_sgd_round():
    """Sec. 4.1's offline reference: worker i follows w <- w - lr * grad on its own batches (the
    update written out here), and since Local SGD only averages at a round's end, the mean of the
    offline models is Local SGD with one round of gamma = steps."""
    bf = _batch_fn(CFG)
    init = wl.init_params(CFG)
    K, lr, steps = CFG["K"], CFG["lr"], 4
    R, losses = oc.s_psgd(init, bf, K, lr, steps)
    assert len(R) == K and len(losses) == steps and len(losses[0]) == K
    for i in range(K):
        w = {k: v.astype(np.float64) for k, v in init.items()}
        for e in range(steps):
            loss, g = oc.loss_and_grads(w, *bf(i, e))
            assert abs(loss - losses[e][i]) <= 1e-12 * abs(loss)
            w = {k: w[k] - lr * g[k] for k in g}
        _close(R[i], w)
    G, _ = oc.s_seq(init, bf, K, lr, gamma=steps, rounds=1)
    _close(G, {k: sum(R[i][k] for i in range(K)) / K for k in init})
    # workers with different batches end up apart
    assert any(np.abs(R[0][k] - R[1][k]).max() > 0 for k in init)


def test_sovl_first_round_applies_nothing_and_update_is_one_round_late():
    """Alg. 3's guard: nothing is applied before the first all-reduce exists; afterwards the
    global model lags the local training by one synchronisation."""
    bf = _batch_fn(CFG)
    init = wl.init_params(CFG)
    K, lr = CFG["K"], CFG["lr"]
    trace = []
    G, _ = oc.s_ovl(init, bf, K, lr, rounds=3, trace=trace)
    i64 = {k: v.astype(np.float64) for k, v in init.items()}
    for k in init:
        assert np.array_equal(trace[0][k], i64[k])
    # round-0 and round-1 deltas are both taken at the initial model
    d = []
    for t in (0, 1):
        reps = [oc.local_step(i64, *bf(k, t), lr)[0] for k in range(K)]
        d.append({n: sum(r[n] - i64[n] for r in reps) / K for n in init})
    _close(trace[1], {n: i64[n] + d[0][n] for n in init})
    g2 = {n: i64[n] + d[0][n] + d[1][n] for n in init}
    _close(trace[2], g2)
    # round 2 trains on init + d0 only
    start2 = {n: i64[n] + d[0][n] for n in init}
    reps = [oc.local_step(start2, *bf(k, 2), lr)[0] for k in range(K)]
    d2 = {n: sum(r[n] - start2[n] for r in reps) / K for n in init}
    _close(G, {n: g2[n] + d2[n] for n in init})


def test_sovl_lr_zero_is_identity():
    init = wl.init_params(CFG)
    G, _ = oc.s_ovl(init, _batch_fn(CFG), CFG["K"], 0.0, rounds=3)
    for k in init:
        assert np.array_equal(G[k], init[k].astype(np.float64))


def test_sovl_quadratic_closed_form():
    """Worker k minimises 0.5*|w - c_k|^2.  With e_t = (start of round t) - mean(c):
    e_{t+1} = e_t - lr * e_{t-1}, e_0 = e_1; solved by the roots of x^2 - x + lr = 0."""
    g = np.random.default_rng(7)
    K, lr, rounds, P = 3, 0.3, 9, 4
    c = [g.standard_normal(P) for _ in range(K)]
    cbar = np.mean(c, axis=0)
    init = {"w": g.standard_normal(P)}
    step = lambda rep, x, y, lr_: ({"w": rep["w"] - lr_ * (rep["w"] - c[x])}, 0.0)
    G, _ = oc.s_ovl(init, lambda k, t: (k, None), K, lr, rounds, step_fn=step)
    l1 = (1 + cmath.sqrt(1 - 4 * lr)) / 2
    l2 = (1 - cmath.sqrt(1 - 4 * lr)) / 2
    e0 = init["w"] - cbar
    # e_t = A l1^t + B l2^t with e_0 = e_1 = e0
    B = (l1 - 1) / (l1 - l2)
    A = 1 - B
    e = lambda t: ((A * l1 ** t + B * l2 ** t).real) * e0
    want = init["w"] + sum(-lr * e(t) for t in range(rounds))
    assert np.abs(G["w"] - want).max() < 1e-12


def test_merge_grad_bruteforce_loops_and_eq1():
    g = np.random.default_rng(3)
    K, P, lr = 3, 6, 0.7
    G = g.standard_normal(P)
    A = [g.standard_normal(P) for _ in range(K)]
    want = np.empty(P)
    for j in range(P):
        tot = 0.0
        for k in range(K):
            tot += A[k][j]
        want[j] = G[j] - lr * tot / K
    assert np.abs(oc.merge_grad(G, A, lr) - want).max() < 1e-15
    assert np.array_equal(oc.merge_grad(G, A, 0.0), G)            # lr = 0: unchanged
    one = oc.merge_grad(G, [A[0]], lr)                            # one worker: a plain SGD step
    assert np.abs(one - (G - lr * A[0])).max() < 1e-15


def test_sseq_in_gradient_form_equals_the_delta_form():
    """Eq. 1 (accumulated gradients) and the delta form `merge` are the same update when the
    learning rate is constant over the round."""
    bf = _batch_fn(CFG)
    init = wl.init_params(CFG)
    K, lr = CFG["K"], CFG["lr"]
    for gamma, rounds in ((1, 3), (3, 2)):
        Gg, lg = oc.s_seq_grad(init, bf, K, lr, gamma, rounds)
        Gd, ld = oc.s_seq(init, bf, K, lr, gamma, rounds)
        _close(Gg, Gd, tol=1e-12)
        assert np.allclose(lg, ld, rtol=1e-12, atol=0)


def test_sasync_with_one_step_per_round_is_sovl():
    bf = _batch_fn(CFG)
    init = wl.init_params(CFG)
    K, lr = CFG["K"], CFG["lr"]
    Ga, la = oc.s_async(init, bf, K, lr, [1, 1, 1, 1])
    Go, lo = oc.s_ovl(init, bf, K, lr, rounds=4)
    for k in init:
        assert np.array_equal(Ga[k], Go[k]), k
    assert la == lo


def test_sasync_single_round_single_worker_is_plain_sgd():
    """One worker, one round of n steps: the merge adds exactly that worker's change."""
    bf = _batch_fn(CFG)
    init = wl.init_params(CFG)
    lr = CFG["lr"]
    G, _ = oc.s_async(init, bf, 1, lr, [3])
    w = {k: v.astype(np.float64) for k, v in init.items()}
    for e in range(3):
        w, _ = oc.local_step(w, *bf(0, e), lr)
    _close(G, w)


def test_sasync_is_alg2_alg3_in_gradient_form():
    """The literal bookkeeping of Alg. 2 / Alg. 3 (accumulated gradients, counter, status, the
    update applied one synchronisation after its all-reduce, Eq. 1 with the mean) on a model
    whose gradient is known in closed form, against the delta form the oracle uses.
    Worker k minimises 0.5*|w - c_k|^2 with plain SGD; `busy` steps after a StartSync find
    the status `synchronizing`."""
    g = np.random.default_rng(11)
    K, lr, P = 3, 0.2, 5
    c = [g.standard_normal(P) for _ in range(K)]
    counts = [1, 3, 2, 1, 4, 2]
    init = {"w": g.standard_normal(P)}
    step = lambda rep, x, y, lr_: ({"w": rep["w"] - lr_ * (rep["w"] - c[x])}, 0.0)
    G, _ = oc.s_async(init, lambda k, t: (k, None), K, lr, counts, step_fn=step)

    # Alg. 2 / Alg. 3 as written, all K workers in lockstep
    w = init["w"].copy()                      # global model
    pending = None                            # all-reduced gradients waiting for the next StartSync
    acc = [np.zeros(P) for _ in range(K)]     # accumulated gradients of the running round
    rep = [w.copy() for _ in range(K)]        # replicas: clone(w) when counter == 0
    for n in counts:
        for k in range(K):
            rep[k] = w.copy()                 # counter == 0: make replica
        for _ in range(n):
            for k in range(K):
                grad = rep[k] - c[k]
                rep[k] = rep[k] - lr * grad   # update replica
                acc[k] = acc[k] + grad        # accumulate gradients
        # status idle: StartSync.  P_s first applies the previous all-reduce, then all-reduces
        if pending is not None:
            w = w - lr * pending
        pending = sum(acc) / K
        acc = [np.zeros(P) for _ in range(K)]
    w = w - lr * pending                      # the last all-reduce, applied by the final sync
    assert np.abs(G["w"] - w).max() < 1e-12


def test_overlap_counts_match_the_worked_example():
    """Sec. 3.2: in the span of one Local-SGD loop, gamma + k + 1 trainings and
    (gamma + 1)/k + 1 synchronisations.  Values for gamma = 8 (Sec. 4.1) in tests/golden."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "overlap_counts.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert rows
    for gamma, k, trains, syncs in rows:
        t, s = oc.overlap_counts(int(gamma), int(k))
        assert t == int(trains)
        assert abs(s - float(syncs)) < 1e-12
