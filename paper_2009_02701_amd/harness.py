"""Device-side driver of the HPSGD schedules over the C-ABI library.

Owns the device buffers (global model, two generations of K replicas and snapshots,
workspace, resident data shards) and enqueues the library calls: batch gather, local
step of all K workers, merge, sync.  Two schedules:

  * s_seq(gamma, rounds): no staleness -- gamma local steps, merge, sync (Local SGD in the
    gradient form of Eq. 1; gamma = 1 is SSGD).
  * s_ovl(rounds): the paper's hierarchy (Sec. 3.1): the synchronising side (stream B) merges
    the previous round's replica changes while the training side (stream A) already runs
    the next local step on the other buffer generation; the global update therefore lands one
    synchronisation late (Sec. 3.2, after Alg. 3).

No arithmetic happens here: torch is used for memory, streams and events only.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as hb


class Trainer:
    def __init__(self, cfg: dict, init_params: dict, shards: list, orders: list, device="cuda",
                 aux_stream=True, prepare=False, implicit_clone=True):
        # Overlapped schedule: "make replica" (Alg. 2) is not a copy of its own.  The synchronising
        # side only takes the snapshot of the merged global model; the local step reads its
        # parameters from that one snapshot and writes the K updated replicas
        # (hpsgd_local_step_all_cloned): the same bits, 4 (K + 1) bytes per parameter less per round.
        self.implicit_clone = implicit_clone
        # hpsgd_prepare_replicas behind every clone on the synchronising side.  Off by default: on
        # MI355X the copies then run beside the training stream's resident-weight launches, whose
        # chains of waits slow down by more than the copies cost (config 3: 3.37 -> 3.60 ms per round)
        self.use_prepare = prepare
        # The synchronising side's merge + clone as one pass (hpsgd_merge_sync: the same bits, 80 instead
        # of 84 bytes per parameter at K = 8).  Off: on MI355X the pass that reads ten streams and writes
        # ten runs at 5.2 TB/s where the read-mostly merge and the write-mostly clone run at 5.8 and
        # 5.4 TB/s, so the two calls take 1.50 ms for 100 M parameters and the one pass 1.52 ms.
        self.fused_merge_sync = False
        self.cfg = cfg
        self.ctx = hb.Context(cfg)
        self.K, self.P, self.stride = self.ctx.K, self.ctx.P, self.ctx.stride
        dev = torch.device(device)
        self.dev = dev
        K, B = self.K, cfg["batch"]
        flat = np.zeros(self.stride, np.float32)
        flat[:self.P] = self.ctx.flatten(init_params)
        self.G = torch.from_numpy(flat).to(dev)
        self.S = [torch.zeros(self.stride, dtype=torch.float32, device=dev) for _ in range(2)]
        self.R = [torch.zeros(K, self.stride, dtype=torch.float32, device=dev) for _ in range(2)]
        self.ws = [self.ctx.new_workspace(dev), None]
        self.loss = torch.zeros(K, dtype=torch.float32, device=dev)
        self.losses = []
        # resident shards and the batch order
        kind = cfg["kind"]
        self.kind = kind
        self.xs = [torch.from_numpy(np.ascontiguousarray(s[0])).to(dev) for s in shards]
        self.ys = [torch.from_numpy(np.ascontiguousarray(s[1])).to(dev) if s[1] is not None else None
                   for s in shards]
        self.order = [torch.from_numpy(np.ascontiguousarray(o)).to(dev) for o in orders]
        self.n_batches = orders[0].size // B
        if kind == "gru_cls":
            T, I = cfg["seq_len"], cfg["input"]
            self.xb = torch.zeros(K, T, B, I, dtype=torch.float32, device=dev)
            self.yb = torch.zeros(K, B, dtype=torch.int32, device=dev)
        elif kind == "mlp":
            self.xb = torch.zeros(K, B, cfg["dims"][0], dtype=torch.float32, device=dev)
            self.yb = torch.zeros(K, B, dtype=torch.int32, device=dev)
        else:
            T = cfg["seq_len"]
            self.xb = torch.zeros(K, T, B, dtype=torch.int32, device=dev)
            self.yb = torch.zeros(K, T, B, dtype=torch.int32, device=dev)
        self.stream_a = torch.cuda.Stream(device=dev)
        self.stream_b = torch.cuda.Stream(device=dev)
        # third stream: weight-gradient GEMMs beside the BPTT recurrence, inside a local step
        self.stream_aux = torch.cuda.Stream(device=dev) if aux_stream else None
        self.ctx.set_aux_stream(self.stream_aux)
        torch.cuda.synchronize(dev)

    # ------------------------------------------------------------------ pieces
    def gather(self, step: int, stream=None):
        """Assemble every worker's mini-batch `step` from its resident shard (bit-exact)."""
        cfg, B, K = self.cfg, self.cfg["batch"], self.K
        s = step % self.n_batches
        idx = [self.order[k][s * B:(s + 1) * B] for k in range(K)]
        xb, yb = list(self.xb), list(self.yb)
        if self.kind == "gru_cls":
            hb.gather_batch_all(self.xs, idx, cfg["seq_len"], cfg["input"], xb, stream=stream)
            hb.gather_batch_all(self.ys, idx, 1, 1, yb, row_elems=1, stream=stream)
        elif self.kind == "mlp":
            hb.gather_batch_all(self.xs, idx, 1, cfg["dims"][0], xb, stream=stream)
            hb.gather_batch_all(self.ys, idx, 1, 1, yb, row_elems=1, stream=stream)
        else:
            T = cfg["seq_len"]
            tok = [x.view(-1) for x in self.xs]
            hb.gather_batch_all(tok, idx, T, 1, xb, row_elems=T + 1, stream=stream)
            hb.gather_batch_all([t[1:] for t in tok], idx, T, 1, yb, row_elems=T + 1, stream=stream)

    def local_step_cloned(self, gen: int, lr: float, stream=None, ws=0):
        """The local step of generation `gen` whose replicas are still clones of its snapshot."""
        if self.ws[ws] is None:
            self.ws[ws] = self.ctx.new_workspace(self.dev)
        self.ctx.local_step_all_cloned(self.S[gen][:self.P], self.R[gen], self.xb, self.yb, lr, self.loss,
                                       self.ws[ws], stream=stream)

    def snapshot(self, gen: int, stream=None):
        """S[gen] = global model (hpsgd_sync_all with no replica to write)."""
        hb.sync_all(self.G[:self.P], [], self.S[gen][:self.P], stream=stream)

    def local_step(self, gen: int, lr: float, stream=None, ws=0):
        if self.ws[ws] is None:
            self.ws[ws] = self.ctx.new_workspace(self.dev)
        self.ctx.local_step_all(self.R[gen], self.R[gen], self.xb, self.yb, lr, self.loss,
                                self.ws[ws], stream=stream)

    def prepare(self, gen: int, stream=None):
        """hpsgd_prepare_replicas for generation `gen`, whose local steps use workspace `gen`."""
        if self.ws[gen] is None:
            self.ws[gen] = self.ctx.new_workspace(self.dev)
        if self.use_prepare == "clones_b":
            # (the snapshot is the clone's source as it was at clone time; the global model moves on)
            self.ctx.prepare_clones(self.S[gen][:self.P], self.R[gen], self.ws[gen], stream=stream, with_head=True)
        elif self.use_prepare is True or self.use_prepare == "replicas_b":
            self.ctx.prepare_replicas(self.R[gen], self.ws[gen], stream=stream)

    def prepare_clones_on_training_stream(self, gen: int, stream=None):
        """The operand copies of freshly cloned replicas, made on the training stream right before the
        local step (which then skips its own) from the generation's snapshot: the global model as it
        was when the replicas were cloned (the global model itself may already have moved on)."""
        if self.use_prepare == "clones_a":
            if self.ws[gen] is None:
                self.ws[gen] = self.ctx.new_workspace(self.dev)
            self.ctx.prepare_clones(self.S[gen][:self.P], self.R[gen], self.ws[gen], stream=stream)

    def merge(self, gen: int, stream=None):
        hb.merge(self.G[:self.P], [self.R[gen][k, :self.P] for k in range(self.K)],
                 self.S[gen][:self.P], stream=stream)

    def merge_snapshot(self, gen: int, stream=None):
        """merge(gen) followed by snapshot(gen) in one pass (the replicas are only read)."""
        hb.merge_snapshot(self.G[:self.P], [self.R[gen][k, :self.P] for k in range(self.K)],
                          self.S[gen][:self.P], stream=stream)

    def merge_sync(self, gen: int, stream=None):
        """merge(gen) followed by sync_all(gen) in one pass over the buffers."""
        hb.merge_sync(self.G[:self.P], [self.R[gen][k, :self.P] for k in range(self.K)],
                      self.S[gen][:self.P], stream=stream)

    def sync_all(self, gen: int, stream=None):
        hb.sync_all(self.G[:self.P], [self.R[gen][k, :self.P] for k in range(self.K)],
                    self.S[gen][:self.P], stream=stream)

    def global_params(self) -> dict:
        torch.cuda.synchronize(self.dev)
        return self.ctx.unflatten(self.G[:self.P].cpu().numpy())

    def replica_params(self, gen: int, k: int) -> dict:
        torch.cuda.synchronize(self.dev)
        return self.ctx.unflatten(self.R[gen][k, :self.P].cpu().numpy())

    # ------------------------------------------------------------------ schedules
    def s_seq(self, lr: float, gamma: int, rounds: int, record_loss=True, sync_delay_us: int = 0):
        """Blocking order (gamma = 1: synchronous SGD; gamma > 1: Local SGD, Alg. 1): the
        synchronisation - and its optional synthetic latency - sits on the training stream."""
        st = self.stream_a
        st.wait_stream(torch.cuda.current_stream())
        step = 0
        have_snapshot = False
        for _ in range(rounds):
            # (the clone is implicit here too: the first local step after a synchronisation reads the
            # snapshot, which the merge of the round before has left behind in the same pass)
            if self.implicit_clone:
                if not have_snapshot:
                    self.snapshot(0, st)
            else:
                self.sync_all(0, st)
            for i in range(gamma):
                self.gather(step, st)
                if self.implicit_clone and i == 0:
                    self.local_step_cloned(0, lr, st)
                else:
                    self.local_step(0, lr, st)
                if record_loss:
                    with torch.cuda.stream(st):
                        self.losses.append(self.loss.clone())
                step += 1
            if sync_delay_us:
                hb.delay_us(sync_delay_us, st)
            if self.implicit_clone:
                self.merge_snapshot(0, st)
                have_snapshot = True
            else:
                self.merge(0, st)
        st.synchronize()

    def s_psgd(self, lr: float, steps: int, record_loss=True):
        """Purely offline training (Sec. 4.1): local steps only, after one initial sync; the K
        replicas never meet.  The reference for the time the training itself takes."""
        st = self.stream_a
        st.wait_stream(torch.cuda.current_stream())
        self.sync_all(0, st)
        for step in range(steps):
            self.gather(step, st)
            self.local_step(0, lr, st)
            if record_loss:
                with torch.cuda.stream(st):
                    self.losses.append(self.loss.clone())
        st.synchronize()

    def s_train_side(self, lr: float, steps: int):
        """The training side of an overlapped round by itself, as that round runs it (gather, the
        operand copies if they are made on this stream, the local step from the snapshot), with
        nothing on the synchronising side: a time reference, not a training schedule."""
        st = self.stream_a
        st.wait_stream(torch.cuda.current_stream())
        if self.implicit_clone:
            self.snapshot(0, st)
        else:
            self.sync_all(0, st)
        for step in range(steps):
            self.gather(step, st)
            if self.implicit_clone:
                self.prepare_clones_on_training_stream(0, st)
                self.local_step_cloned(0, lr, st)
            else:
                self.local_step(0, lr, st)
        st.synchronize()

    def s_ovl(self, lr: float, rounds: int, record_loss=True, single_stream=False):
        """Overlapped schedule; with single_stream=True the same op list runs on one stream."""
        self.ovl_begin(single_stream)
        for t in range(rounds):
            self.ovl_round(t, lr, record_loss)
        self.ovl_drain()

    def s_seq_grad(self, lr: float, gamma: int, rounds: int, record_loss=True):
        """s_seq with the synchronisation in gradient form (Eq. 1 as printed): the workers
        accumulate their gradients over a round, the global model moves by -lr * their mean."""
        st = self.stream_a
        st.wait_stream(torch.cuda.current_stream())
        if self.ws[0] is None:
            self.ws[0] = self.ctx.new_workspace(self.dev)
        with torch.cuda.stream(st):
            acc = torch.zeros_like(self.R[0])
        step = 0
        for _ in range(rounds):
            self.sync_all(0, st)
            with torch.cuda.stream(st):
                acc.zero_()
            for _ in range(gamma):
                self.gather(step, st)
                self.ctx.local_step_all_acc(self.R[0], self.R[0], self.xb, self.yb, lr, self.loss, acc,
                                            self.ws[0], stream=st)
                if record_loss:
                    with torch.cuda.stream(st):
                        self.losses.append(self.loss.clone())
                step += 1
            hb.merge_grad(self.G[:self.P], [acc[k, :self.P] for k in range(self.K)], lr, stream=st)
        st.synchronize()

    def s_async(self, lr: float, epochs: int, sync_delay_us: int = 0, record_loss=False):
        """Alg. 2 + Alg. 3 with the status check made at run time: after every local step the
        training side (stream A) asks, without waiting, whether the synchronising side
        (stream B) is idle.  If it is, the generation just trained is handed over (StartSync:
        merge of its replica changes, then a fresh clone of the global model) and training
        goes on at once on the other generation; if not, the next local step stays on the
        same generation.  Returns the number of local steps of every round - what the
        float64 oracle needs to replay the run.  sync_delay_us: extra time the synchronising
        side takes per round (a slow interconnect).  At most two local steps are in flight, so
        the status the host reads is the one the device is in."""
        sa, sb = self.stream_a, self.stream_b
        sa.wait_stream(torch.cuda.current_stream())
        # (implicit clones: a generation's first local step after its synchronisation reads the snapshot)
        clone = self.snapshot if self.implicit_clone else self.sync_all
        clone(0, sa)
        clone(1, sa)
        fresh = [self.implicit_clone, self.implicit_clone]
        g, n, counts = 0, 0, []
        busy = None  # event: the synchronising side's running job
        done = [torch.cuda.Event(), torch.cuda.Event()]
        for e in range(epochs):
            if e >= 2:
                done[e % 2].synchronize()
            self.gather(e, sa)
            if fresh[g]:
                self.local_step_cloned(g, lr, sa, ws=g)
                fresh[g] = False
            else:
                self.local_step(g, lr, sa, ws=g)
            n += 1
            if record_loss:
                with torch.cuda.stream(sa):
                    self.losses.append(self.loss.clone())
            done[e % 2].record(sa)
            if busy is None or busy.query():  # status == idle
                sb.wait_event(done[e % 2])
                if sync_delay_us:
                    hb.delay_us(sync_delay_us, sb)
                if self.implicit_clone:
                    self.merge_snapshot(g, sb)
                elif self.fused_merge_sync:
                    self.merge_sync(g, sb)
                else:
                    self.merge(g, sb)
                    clone(g, sb)
                fresh[g] = self.implicit_clone
                self.prepare(g, sb)
                busy = torch.cuda.Event()
                busy.record(sb)
                counts.append(n)
                g, n = 1 - g, 0
        if busy is not None:
            sa.wait_event(busy)
        if n:
            self.merge(g, sa)
            counts.append(n)
        sa.synchronize()
        sb.synchronize()
        return counts

    def ovl_begin(self, single_stream=False):
        self._sa = self.stream_a
        self._sb = self.stream_a if single_stream else self.stream_b
        self._sa.wait_stream(torch.cuda.current_stream())
        if self.implicit_clone:
            self.snapshot(0, self._sa)
        else:
            self.sync_all(0, self._sa)
        self._g = 0
        self._ev_a = torch.cuda.Event()
        self._ev_b = torch.cuda.Event()
        self._ev_a.record(self._sa)
        self._have_delta = False

    def ovl_round(self, t: int, lr: float, record_loss=False):
        sa, sb, g = self._sa, self._sb, self._g
        # synchronising side (stream B): merge the previous round's replica changes, once the
        # local step that produced them (and the clone after it) is done
        # ... and clone the global model into that generation for the next round ("make replica"):
        # it depends on the merge only, so it sits behind it on the synchronising side and off
        # the training stream's path; merge and clone of one generation are one pass (the same bits)
        clone = self.snapshot if self.implicit_clone else self.sync_all
        if self._have_delta:
            sb.wait_event(self._ev_a)
            if self.implicit_clone:
                self.merge_snapshot(1 - g, sb)
            elif self.fused_merge_sync:
                self.merge_sync(1 - g, sb)
            else:
                self.merge(1 - g, sb)
                clone(1 - g, sb)
        else:
            clone(1 - g, sb)
        # ... and the operand copies of its weights that the next local step would make at its
        # start (bf16 configurations), in that generation's own workspace
        self.prepare(1 - g, sb)
        self._ev_b.record(sb)
        # training side (stream A): this round's local step on generation g
        self.gather(t, sa)
        self.prepare_clones_on_training_stream(g, sa)
        if self.implicit_clone:
            self.local_step_cloned(g, lr, sa, ws=g)
        else:
            self.local_step(g, lr, sa, ws=g)
        if record_loss:
            with torch.cuda.stream(sa):
                self.losses.append(self.loss.clone())
        # boundary: the next round's local step waits for B's merge and clone
        self._ev_a.record(sa)
        sa.wait_event(self._ev_b)
        self._g = 1 - g
        self._have_delta = True

    # ------------------------------------------------------------------ overlapped rounds as a HIP graph
    def ovl_capture(self, t0: int, lr: float):
        """Captures the next `period` overlapped rounds (starting at round t0, which must continue an
        ovl_begin / ovl_round sequence with at least two rounds behind it) into one HIP graph and
        returns it; period = lcm(2 buffer generations, batches per shard), after which the rounds'
        arguments repeat, so every replay issues the rounds t0 + i * period ... of the schedule.
        The host then launches one graph per `period` rounds instead of some twenty to forty kernels
        per round.  The two side streams (synchronising, auxiliary) join the capture through the
        events the schedule records anyway, and every round ends with the training stream waiting
        for the synchronising one, so the capture closes on the training stream alone.
        Nothing in the rounds is a memset (cleared memory is cleared by kernels), and nothing
        allocates."""
        assert self._have_delta and self._sb is not self._sa
        period = self.n_batches if self.n_batches % 2 == 0 else 2 * self.n_batches
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize(self.dev)
        with torch.cuda.stream(self._sa):
            graph.capture_begin(capture_error_mode="thread_local")
            try:
                # the event the synchronising stream waits for at the start of a round, recorded anew
                # inside the capture: a wait for the one recorded before it would tie the graph to
                # work outside it (everything before the capture precedes the graph on this stream)
                self._ev_a.record(self._sa)
                for i in range(period):
                    self.ovl_round(t0 + i, lr)
            finally:
                graph.capture_end()
        self._graph_period = period
        return graph

    def ovl_replay(self, graph):
        """One replay = `period` rounds (see ovl_capture), issued on the training stream."""
        with torch.cuda.stream(self._sa):
            graph.replay()
        return self._graph_period

    def ovl_drain(self):
        if self._have_delta:
            self.merge(1 - self._g, self._sa)
            self._have_delta = False
        self._sa.synchronize()
        self._sb.synchronize()
