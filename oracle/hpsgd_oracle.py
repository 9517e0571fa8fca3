"""CPU oracle for the HPSGD hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 numpy statement of what the hot path computes: the local
training step of one worker (forward, backprop through time, SGD commit to the
worker's replica), the replica merge and the replica sync, plus the two
schedules that chain them.  Only the tests, the smoke check and the benchmark's
cpu_baseline leg may import it; the product path never does.  It shares no code
with the HIP path and takes no value from it.

What fixes each function:
  * commit        -- Alg. 2, "update replica": r_i <- r_i - mu * grad.
  * merge         -- Eq. 1 with Alg. 3's all-reduce read as a mean over the n
                     workers: W <- W_prev - mu * sum_i sum_e grad_i^e / n, written
                     with replica_k - snapshot = -mu * (accumulated gradients of k).
  * sync          -- Alg. 2, "make replica": r_i <- clone(w).
  * gather_batch  -- Sec. 3.2, a worker's mini-batch out of its own sub-dataset (exact copies).
  * model forward / backward -- the paper names a GRU (Sec. 1) and cross-entropy
                     with plain SGD (Sec. 4.1) but prints no model equations; the
                     cell is the one of the library the paper ran on (gate order
                     r, z, n; two bias vectors; candidate n = tanh(W_in x + b_in +
                     r * (W_hn h + b_hn)); h_0 = 0), loss = mean cross-entropy.
  * schedules     -- Sec. 3.1/3.2: s_seq is the no-staleness order (Local SGD,
                     Alg. 1, by Eq. 2); s_ovl applies each merge one round late,
                     the one-synchronisation delay stated after Alg. 3.

Pins (tests/test_oracle_*.py): a hand-written mini-batch for gather_batch; central finite differences of every parameter,
a double-precision library GRU with autograd, the T=1 closed form, loss = ln C at
zero weights, Eq. 2, K identical replicas, K=1 == plain SGD, lr=0, SSGD and
Local-SGD equivalences, a closed-form delayed recursion on a quadratic.
Absolute task accuracy (the paper's accuracy curves): parity unpinned -- those
need the paper's dataset and CNNs and are not part of this path.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _f64(params: dict) -> dict:
    return {k: np.asarray(v, dtype=F64).copy() for k, v in params.items()}


def _mm(a, b, rnd):
    """Matrix product; `rnd` (None = exact float64) models operand rounding: a test may pass a
    function that rounds every GEMM operand to a narrower format before the product."""
    return a @ b if rnd is None else rnd(a) @ rnd(b)


def sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


# ----------------------------------------------------------------------------
# softmax cross-entropy, mean over rows
# ----------------------------------------------------------------------------
def softmax_ce(logits, y):
    """loss = mean_i -log softmax(logits_i)[y_i];  returns (loss, dloss/dlogits)."""
    n = logits.shape[0]
    m = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - m)
    s = e.sum(axis=1, keepdims=True)
    p = e / s
    logp = (logits - m) - np.log(s)
    loss = -logp[np.arange(n), y].mean()
    d = p.copy()
    d[np.arange(n), y] -= 1.0
    return loss, d / n


# ----------------------------------------------------------------------------
# one GRU layer
# ----------------------------------------------------------------------------
def gru_layer_forward(W_ih, W_hh, b_ih, b_hh, x, rnd=None):
    """x [T,B,in] -> hs [T+1,B,H] (hs[0] = 0, hs[t+1] = h after step t) and saved gates."""
    T, B, _ = x.shape
    H = W_hh.shape[1]
    hs = np.zeros((T + 1, B, H), F64)
    r = np.zeros((T, B, H), F64)
    z = np.zeros((T, B, H), F64)
    n = np.zeros((T, B, H), F64)
    q = np.zeros((T, B, H), F64)
    for t in range(T):
        gx = _mm(x[t], W_ih.T, rnd) + b_ih
        gh = _mm(hs[t], W_hh.T, rnd) + b_hh
        r[t] = sigmoid(gx[:, 0:H] + gh[:, 0:H])
        z[t] = sigmoid(gx[:, H:2 * H] + gh[:, H:2 * H])
        q[t] = gh[:, 2 * H:3 * H]
        n[t] = np.tanh(gx[:, 2 * H:3 * H] + r[t] * q[t])
        hs[t + 1] = (1.0 - z[t]) * n[t] + z[t] * hs[t]
    return hs, (r, z, n, q)


def gru_layer_backward(W_ih, W_hh, x, hs, saved, dh_out, rnd=None):
    """dh_out [T,B,H]: dLoss/d(h_t) arriving from above at every step.

    Returns dW_ih, dW_hh, db_ih, db_hh, dx [T,B,in].
    """
    r, z, n, q = saved
    T, B, _ = x.shape
    H = W_hh.shape[1]
    dW_ih = np.zeros_like(W_ih)
    dW_hh = np.zeros_like(W_hh)
    db_ih = np.zeros(3 * H, F64)
    db_hh = np.zeros(3 * H, F64)
    dx = np.zeros_like(x)
    dh_next = np.zeros((B, H), F64)
    for t in range(T - 1, -1, -1):
        dh = dh_out[t] + dh_next
        h_prev = hs[t]
        dn = dh * (1.0 - z[t])
        dz = dh * (h_prev - n[t])
        da_n = dn * (1.0 - n[t] ** 2)
        dr = da_n * q[t]
        dq = da_n * r[t]
        da_r = dr * r[t] * (1.0 - r[t])
        da_z = dz * z[t] * (1.0 - z[t])
        dgx = np.concatenate([da_r, da_z, da_n], axis=1)
        dgh = np.concatenate([da_r, da_z, dq], axis=1)
        dW_ih += _mm(dgx.T, x[t], rnd)
        dW_hh += _mm(dgh.T, h_prev, rnd)
        db_ih += dgx.sum(axis=0)
        db_hh += dgh.sum(axis=0)
        dx[t] = _mm(dgx, W_ih, rnd)
        dh_next = dh * z[t] + _mm(dgh, W_hh, rnd)
    return dW_ih, dW_hh, db_ih, db_hh, dx


# ----------------------------------------------------------------------------
# whole models: loss and gradient of every parameter
# ----------------------------------------------------------------------------
def _n_layers(params):
    l = 0
    while f"l{l}.W_ih" in params:
        l += 1
    return l


def gru_loss_and_grads(params, x, y, rnd=None):
    """GRU classifier (x float [T,B,I], y int [B], head on the last hidden state) or
    GRU language model (x int [T,B] token ids, y int [T,B] next tokens, head at every step;
    recognised by the presence of an embedding table)."""
    p = _f64(params)
    L = _n_layers(p)
    lm = "embed.E" in p
    if lm:
        tokens = np.asarray(x)
        inp = p["embed.E"][tokens]          # [T,B,E]
    else:
        inp = np.asarray(x, F64)
    T, B = inp.shape[0], inp.shape[1]
    layer_in, layer_hs, layer_saved = [], [], []
    for l in range(L):
        hs, saved = gru_layer_forward(p[f"l{l}.W_ih"], p[f"l{l}.W_hh"],
                                      p[f"l{l}.b_ih"], p[f"l{l}.b_hh"], inp, rnd)
        layer_in.append(inp)
        layer_hs.append(hs)
        layer_saved.append(saved)
        inp = hs[1:]
    top = layer_hs[-1]
    H = top.shape[2]
    Wo, bo = p["head.W"], p["head.b"]
    g = {}
    dh_out = np.zeros((T, B, H), F64)
    if lm:
        feats = top[1:].reshape(T * B, H)
        logits = _mm(feats, Wo.T, rnd) + bo
        loss, dlog = softmax_ce(logits, np.asarray(y).reshape(T * B))
        g["head.W"] = _mm(dlog.T, feats, rnd)
        g["head.b"] = dlog.sum(axis=0)
        dh_out = _mm(dlog, Wo, rnd).reshape(T, B, H)
    else:
        feats = top[T]
        logits = _mm(feats, Wo.T, rnd) + bo
        loss, dlog = softmax_ce(logits, np.asarray(y))
        g["head.W"] = _mm(dlog.T, feats, rnd)
        g["head.b"] = dlog.sum(axis=0)
        dh_out[T - 1] = _mm(dlog, Wo, rnd)
    for l in range(L - 1, -1, -1):
        dW_ih, dW_hh, db_ih, db_hh, dx = gru_layer_backward(
            p[f"l{l}.W_ih"], p[f"l{l}.W_hh"], layer_in[l], layer_hs[l], layer_saved[l], dh_out, rnd)
        g[f"l{l}.W_ih"], g[f"l{l}.W_hh"] = dW_ih, dW_hh
        g[f"l{l}.b_ih"], g[f"l{l}.b_hh"] = db_ih, db_hh
        dh_out = dx
    if lm:
        dE = np.zeros_like(p["embed.E"])
        np.add.at(dE, tokens.reshape(-1), dh_out.reshape(T * B, -1))
        g["embed.E"] = dE
    return loss, g


def mlp_loss_and_grads(params, x, y, rnd=None, flip=()):
    """ReLU MLP, x float [B,D0], y int [B]; ReLU'(0) = 0.

    flip: (layer i, sample b, unit j) triples of hidden units whose ReLU takes the OTHER branch in
    the backward pass.  For a pre-activation within rounding of zero the branch is decided by the
    last bits of a sum, so an fp32 implementation may land on either side; a test that finds such
    units (mlp_preactivations) may accept either branch for them.  Empty by default."""
    p = _f64(params)
    L = 0
    while f"fc{L}.W" in p:
        L += 1
    acts = [np.asarray(x, F64)]
    for i in range(L):
        a = _mm(acts[-1], p[f"fc{i}.W"].T, rnd) + p[f"fc{i}.b"]
        if i < L - 1:
            a = np.maximum(a, 0.0)
        acts.append(a)
    masks = [acts[i] > 0.0 for i in range(L)]
    for (i, b, j) in flip:
        masks[i + 1][b, j] = not masks[i + 1][b, j]
    loss, delta = softmax_ce(acts[-1], np.asarray(y))
    g = {}
    for i in range(L - 1, -1, -1):
        g[f"fc{i}.W"] = _mm(delta.T, acts[i], rnd)
        g[f"fc{i}.b"] = delta.sum(axis=0)
        if i > 0:
            delta = _mm(delta, p[f"fc{i}.W"], rnd) * masks[i]
    return loss, g


def mlp_preactivations(params, x):
    """The hidden layers' pre-activations a_i = h_{i-1} W_i^T + b_i (before the ReLU), i = 0 .. L-2."""
    p = _f64(params)
    out, h, i = [], np.asarray(x, F64), 0
    while f"fc{i + 1}.W" in p:
        a = h @ p[f"fc{i}.W"].T + p[f"fc{i}.b"]
        out.append(a)
        h = np.maximum(a, 0.0)
        i += 1
    return out


def loss_and_grads(params, x, y, rnd=None):
    if "fc0.W" in params:
        return mlp_loss_and_grads(params, x, y, rnd)
    return gru_loss_and_grads(params, x, y, rnd)


# ----------------------------------------------------------------------------
# the three primitives
# ----------------------------------------------------------------------------
def commit(replica, grads, lr):
    """Alg. 2 'update replica': r <- r - mu * grad, every parameter, plain SGD."""
    return {k: np.asarray(replica[k], F64) - lr * grads[k] for k in replica}


def local_step(replica, x, y, lr):
    """Forward + backward on the replica's parameters, then the commit.  Returns (replica', loss)."""
    loss, g = loss_and_grads(replica, x, y)
    return commit(replica, g, lr), loss


def merge(global_, replicas, snapshot):
    """Eq. 1 in delta form: global <- global + (1/K) * sum_k (replica_k - snapshot).

    Works on dicts of tensors or on plain arrays.
    """
    if isinstance(global_, dict):
        return {k: merge(global_[k], [r[k] for r in replicas], snapshot[k]) for k in global_}
    K = len(replicas)
    acc = np.zeros_like(np.asarray(global_, F64))
    for r in replicas:
        acc = acc + (np.asarray(r, F64) - np.asarray(snapshot, F64))
    return np.asarray(global_, F64) + acc / K


def merge_grad(global_, accs, lr):
    """Eq. 1 as printed: the global model moves by -lr times the mean over the workers of their
    accumulated gradients (Alg. 3: all-reduce of the accumulators, then the update)."""
    if isinstance(global_, dict):
        return {k: merge_grad(global_[k], [a[k] for a in accs], lr) for k in global_}
    K = len(accs)
    tot = np.zeros_like(np.asarray(global_, F64))
    for a in accs:
        tot = tot + np.asarray(a, F64)
    return np.asarray(global_, F64) - lr * (tot / K)


def local_step_acc(replica, acc, x, y, lr):
    """Alg. 2, both bookkeeping lines of a local step: update the replica with the step's
    gradient and add the same gradient to the accumulator.  Returns (replica', acc', loss)."""
    loss, g = loss_and_grads(replica, x, y)
    return commit(replica, g, lr), {k: np.asarray(acc[k], F64) + g[k] for k in g}, loss


def sync(global_):
    """Alg. 2 'make replica': an exact copy of the global model."""
    if isinstance(global_, dict):
        return {k: np.array(v, copy=True) for k, v in global_.items()}
    return np.array(global_, copy=True)


def gather_batch(kind, samples, labels, idx):
    """A worker's mini-batch, assembled from its own sub-dataset (Sec. 3.2: every worker trains on
    its sub-dataset) by the sample numbers `idx`, in the layouts the local step takes.  Plain
    element-by-element copies: the result is exact, whatever the element type.

      kind "gru_cls": samples [N, T, I], labels [N] -> x [T, B, I] (time-major), y [B]
      kind "mlp":     samples [N, D],    labels [N] -> x [B, D],                 y [B]
      kind "gru_lm":  samples [N, T+1] token ids (labels unused): a sample is a run of T+1 tokens,
                      its inputs are the first T and its targets the same run one token later
                                                   -> x [T, B], y [T, B]
    """
    samples = np.asarray(samples)
    B = len(idx)
    if kind == "gru_cls":
        _, T, I = samples.shape
        x = np.empty((T, B, I), samples.dtype)
        y = np.empty((B,), np.asarray(labels).dtype)
        for b in range(B):
            for t in range(T):
                x[t, b, :] = samples[idx[b], t, :]
            y[b] = labels[idx[b]]
        return x, y
    if kind == "mlp":
        x = np.empty((B, samples.shape[1]), samples.dtype)
        y = np.empty((B,), np.asarray(labels).dtype)
        for b in range(B):
            x[b, :] = samples[idx[b], :]
            y[b] = labels[idx[b]]
        return x, y
    if kind == "gru_lm":
        T = samples.shape[1] - 1
        x = np.empty((T, B), samples.dtype)
        y = np.empty((T, B), samples.dtype)
        for b in range(B):
            for t in range(T):
                x[t, b] = samples[idx[b], t]
                y[t, b] = samples[idx[b], t + 1]
        return x, y
    raise ValueError(kind)


# ----------------------------------------------------------------------------
# schedules
# ----------------------------------------------------------------------------
def s_seq(init, batch_fn, K, lr, gamma, rounds, step_fn=None):
    """No-staleness order: `rounds` x { gamma local steps on every worker; merge; sync }.

    batch_fn(worker, step) -> (x, y).  step_fn defaults to local_step (a test may pass
    another per-worker update with the same signature).  Returns (global, losses[step][worker]).
    """
    step_fn = step_fn or local_step
    G = _f64(init)
    losses = []
    step = 0
    for _ in range(rounds):
        S = sync(G)
        R = [sync(G) for _ in range(K)]
        for _ in range(gamma):
            row = []
            for k in range(K):
                R[k], loss = step_fn(R[k], *batch_fn(k, step), lr)
                row.append(loss)
            losses.append(row)
            step += 1
        G = merge(G, R, S)
    return G, losses


def s_psgd(init, batch_fn, K, lr, steps):
    """Purely offline training (Sec. 4.1, "Methods": the reference for training speed): every
    worker starts from the initial model and takes `steps` local steps on its own batches; nothing
    is ever exchanged.  Returns (the K local models, losses[step][worker])."""
    R = [sync(_f64(init)) for _ in range(K)]
    losses = []
    for step in range(steps):
        row = []
        for k in range(K):
            R[k], loss = local_step(R[k], *batch_fn(k, step), lr)
            row.append(loss)
        losses.append(row)
    return R, losses


def s_seq_grad(init, batch_fn, K, lr, gamma, rounds):
    """s_seq with the synchronisation in gradient form (what Alg. 2 / Alg. 3 put on the wire):
    every worker accumulates its gradients over the round, the global model is updated with
    Eq. 1.  For a learning rate that is constant over the round this is the delta form of
    `merge` up to rounding.  Returns (global, losses[step][worker])."""
    G = _f64(init)
    losses = []
    step = 0
    for _ in range(rounds):
        R = [sync(G) for _ in range(K)]
        A = [{k: np.zeros_like(v) for k, v in G.items()} for _ in range(K)]
        for _ in range(gamma):
            row = []
            for k in range(K):
                R[k], A[k], loss = local_step_acc(R[k], A[k], *batch_fn(k, step), lr)
                row.append(loss)
            losses.append(row)
            step += 1
        G = merge_grad(G, A, lr)
    return G, losses


def s_ovl(init, batch_fn, K, lr, rounds, step_fn=None, trace=None):
    """Overlapped order: the merge of round t-1 runs beside the local step of round t.

    Two buffer generations g in {0,1}.  Round t trains generation g (cloned from the
    global model at the end of round t-1, i.e. holding merges <= t-2); meanwhile the
    other generation's delta (round t-1) is merged.  The first round merges nothing,
    the last delta is merged in a drain step.  If `trace` is a list, the global model
    as it stands at the end of every round is appended to it.  Returns (global, losses).
    """
    step_fn = step_fn or local_step
    G = _f64(init)
    S = [sync(G), None]
    R = [[sync(G) for _ in range(K)], None]
    g = 0
    losses = []
    for t in range(rounds):
        row = []
        for k in range(K):
            R[g][k], loss = step_fn(R[g][k], *batch_fn(k, t), lr)
            row.append(loss)
        losses.append(row)
        if t > 0:
            G = merge(G, R[1 - g], S[1 - g])
        if trace is not None:
            trace.append(sync(G))
        S[1 - g] = sync(G)
        R[1 - g] = [sync(G) for _ in range(K)]
        g = 1 - g
    G = merge(G, R[1 - g], S[1 - g])
    return G, losses


def s_async(init, batch_fn, K, lr, counts, step_fn=None):
    """Alg. 2 + Alg. 3 with the number of local steps per synchronisation left to the run:
    counts[r] local steps are made while the synchronisation of round r-1 is in flight
    (Sec. 3.1: the training process keeps training as long as `status` is `synchronizing`,
    and starts the next synchronisation as soon as it finds `status` idle).

    Two replica generations alternate.  Round r trains one generation for counts[r] steps
    (mini-batch index = running step number e); its accumulated change is folded into the
    global model and the generation is cloned again, while round r+1 already trains the
    other generation - which was cloned before round r's change existed.  That is the
    one-synchronisation delay of Alg. 3.  counts = [1]*R is s_ovl.  Returns (global, losses).
    """
    step_fn = step_fn or local_step
    G = _f64(init)
    S = [sync(G), sync(G)]
    R = [[sync(G) for _ in range(K)], [sync(G) for _ in range(K)]]
    g = 0
    e = 0
    losses = []
    for n in counts:
        for _ in range(n):
            row = []
            for k in range(K):
                R[g][k], loss = step_fn(R[g][k], *batch_fn(k, e), lr)
                row.append(loss)
            losses.append(row)
            e += 1
        G = merge(G, R[g], S[g])
        S[g] = sync(G)
        R[g] = [sync(G) for _ in range(K)]
        g = 1 - g
    return G, losses


def overlap_counts(gamma, k):
    """Sec. 3.2 worked example: with t_sync = k * t_train, one Local-SGD loop (gamma local
    steps, one more training pass, one synchronisation) lasts (gamma + 1 + k) * t_train.
    In that time a worker that never waits trains gamma + k + 1 times and, synchronising
    back to back, completes (gamma + 1) / k + 1 synchronisations.  Returns (trainings, syncs)."""
    span = (gamma + 1) + k           # in units of t_train
    return span, span / k
