"""Time-based model aggregation on one GPU (Alg. 1 and Alg. 2 of the paper).

The paper's server and trainers are processes on several machines; here the
M trainers are M HIP streams of one GPU (time-sliced by the hardware), the
server is this host thread, the aggregation operator phi is one kernel
(``tma_average``) and the key-value flags are host variables.  Ordering between
a trainer's last step, the averaging and the trainer's next step is expressed
with events, so nothing in a round waits on the host except the server's own
"weights received" point of the timed mode.

Two triggers:
  * every ``n`` local steps per trainer (deterministic; used for parity), and
  * wall clock: aggregate once ``now - T_agg >= dt_int``; each trainer joins at
    its next step boundary, so trainers of different speed contribute different
    numbers of steps (the paper's motivation for a time-based interval).
    T_agg is reset when the averaged weights have been handed back (the listing
    in the paper never updates it; without the reset every poll after the first
    interval would aggregate).
"""
from __future__ import annotations

import time

import torch

from . import binding as B


class AggregationTrigger:
    """Host-side decision logic of Alg. 1 (no GPU involved; the clock is injectable)."""

    def __init__(self, dt_int: float, dt_train: float, clock=time.perf_counter):
        if dt_int <= 0:
            raise ValueError("dt_int must be positive")
        self.dt_int, self.dt_train, self.clock = dt_int, dt_train, clock
        self.t_start = self.t_agg = clock()
        self.rounds = 0

    def should_aggregate(self) -> bool:
        return self.clock() - self.t_agg >= self.dt_int

    def mark_aggregated(self):
        """Call when the averaged weights are back with the trainers."""
        self.t_agg = self.clock()
        self.rounds += 1

    def should_stop(self) -> bool:
        return self.clock() - self.t_start > self.dt_train


class ModelAggregation:
    """M local trainers on M streams with on-device parameter averaging."""

    def __init__(self, trainers, active_mask: int | None = None, record_rounds: int = 0):
        """``record_rounds`` > 0 keeps, for the first that many aggregations, every trainer's parameters as they are
        on the aggregation stream right before and right after phi (``rec_before`` / ``rec_after`` [round, trainer,
        n_params]) and the mean (``rec_global``): copies enqueued on that stream, for checking the ordering."""
        if not trainers:
            raise B.TmaError("ModelAggregation: no trainers")
        n = trainers[0].n_params
        if any(t.n_params != n for t in trainers):
            raise B.TmaError("ModelAggregation: trainers must share one model shape")
        self.trainers = list(trainers)
        self.M = len(trainers)
        self.active_mask = (1 << self.M) - 1 if active_mask is None else active_mask
        dev = trainers[0].W.device
        self.agg_stream = torch.cuda.Stream(device=dev)
        self.ptr_table = torch.tensor([t.W.data_ptr() for t in trainers], dtype=torch.int64, device=dev)
        self.W_global = torch.empty(n, dtype=torch.float32, device=dev)
        self.done = [torch.cuda.Event() for _ in trainers]
        self.agg_done = torch.cuda.Event()
        self.history = []   # steps finished by each trainer at every aggregation
        self.record_rounds = int(record_rounds)
        if self.record_rounds > 0:
            self.rec_before = torch.zeros((self.record_rounds, self.M, n), dtype=torch.float32, device=dev)
            self.rec_after = torch.zeros_like(self.rec_before)
            self.rec_global = torch.zeros((self.record_rounds, n), dtype=torch.float32, device=dev)
        torch.cuda.synchronize(dev)   # uploads and initial weights are in place before the streams start

    def _active(self, i: int) -> bool:
        return bool((self.active_mask >> i) & 1)

    def aggregate(self):
        """Average the active trainers' weights after their enqueued steps and hand the result back."""
        for i, t in enumerate(self.trainers):
            if self._active(i):
                self.done[i].record(t.stream)
                self.agg_stream.wait_event(self.done[i])
        r = len(self.history)
        rec = r < self.record_rounds
        if rec:
            with torch.cuda.stream(self.agg_stream):
                for i, t in enumerate(self.trainers):
                    self.rec_before[r, i].copy_(t.W)
        B.tma_average([t.W for t in self.trainers], active_mask=self.active_mask, W_global_out=self.W_global,
                      ptr_table=self.ptr_table, stream=self.agg_stream)
        if rec:
            with torch.cuda.stream(self.agg_stream):
                for i, t in enumerate(self.trainers):
                    self.rec_after[r, i].copy_(t.W)
                self.rec_global[r].copy_(self.W_global)
        self.agg_done.record(self.agg_stream)
        for i, t in enumerate(self.trainers):
            if self._active(i):
                t.stream.wait_event(self.agg_done)
        self.history.append([t.steps_done for t in self.trainers])

    def run_rounds(self, n_rounds: int, steps_per_round: int, lr: float):
        """Deterministic schedule: every active trainer does ``steps_per_round`` steps, then phi."""
        for _ in range(n_rounds):
            for _ in range(steps_per_round):          # interleaved so that the streams really time-slice
                for i, t in enumerate(self.trainers):
                    if self._active(i):
                        t.step(lr)
            self.aggregate()
        return self.history

    def run_timed(self, dt_int: float, dt_train: float, lr: float, clock=time.perf_counter, max_in_flight: int = 2):
        """Alg. 1 with a wall-clock interval.  The host keeps at most ``max_in_flight`` steps queued per
        trainer, so that "the step a trainer is in when the flag goes up" is well defined."""
        trig = AggregationTrigger(dt_int, dt_train, clock)
        pending = [[] for _ in self.trainers]
        while not trig.should_stop():
            if trig.should_aggregate():
                self.aggregate()
                self.agg_done.synchronize()           # the server has received and returned the weights
                for q in pending:
                    q.clear()
                trig.mark_aggregated()
                continue
            progressed = False
            for i, t in enumerate(self.trainers):
                if not self._active(i):
                    continue
                q = pending[i]
                while q and q[0].query():
                    q.pop(0)
                if len(q) < max_in_flight:
                    t.step(lr)
                    ev = torch.cuda.Event()
                    ev.record(t.stream)
                    q.append(ev)
                    progressed = True
            if not progressed:
                time.sleep(0)                          # every queue is full: yield, the GPU is busy
        for t in self.trainers:
            t.stream.synchronize()
        return self.history

    def synchronize(self):
        for t in self.trainers:
            t.stream.synchronize()
        self.agg_stream.synchronize()
