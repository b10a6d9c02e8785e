"""Replays an event list (see the harness's scenario description) on the CPU oracle.
TEST INFRASTRUCTURE ONLY; never imported by the product path."""
from __future__ import annotations

from typing import Callable, Dict, Iterator, List, Tuple

import numpy as np

from . import oracle as orc


class OracleReplay:
    def __init__(self, scenario, data_seed: int, dropout_seed: int, theta0: np.ndarray, minibatches: Callable,
                 dropout_p: float = 0.25, dims: orc.Dims = orc.Dims(), n_threads: int = 0, eval_batch: Callable = None):
        """`minibatches(data_seed, mb_ids, batch)` and `eval_batch(data_seed, eval_id, n_images)` are the
        harness's input generators."""
        self.eval_batch = eval_batch
        self.evals: List[tuple] = []         # (eval_id, loss, accuracy, predictions, logits)
        self.dropped: List[int] = []
        self.sc = scenario
        self.data_seed = data_seed
        self.minibatches = minibatches
        self.server = orc.OracleServer(dims, seed=dropout_seed, dropout_p=dropout_p, n_slots=scenario.n_slots,
                                       theta=theta0, n_threads=n_threads)
        self.meta_log: List[tuple] = []
        self.last: Dict[int, orc.QueueEntry] = {}     # entries appended by the most recent "grads" event
        self.losses: Dict[int, float] = {}

    def steps(self) -> Iterator[Tuple[tuple, List[int]]]:
        """Executes the events one by one; yields (event, arrival numbers it appended) after each."""
        sv = self.server
        for ev in self.sc.events:
            kind, seqs = ev[0], []
            if kind == "grads":
                _, workers, slots, mbs = ev
                x, y = self.minibatches(self.data_seed, mbs, self.sc.batch)
                self.last = {}
                for e in sv.worker_grads_batched(workers, slots, mbs, x, y):
                    self.meta_log.append((e.seq, e.worker, e.version, e.mb_id))
                    self.losses[e.seq] = e.loss
                    self.last[e.seq] = e
                    seqs.append(e.seq)
            elif kind == "sync":
                sv.apply_sync(ev[1], ev[2])
            elif kind == "async":
                sv.apply_async(ev[1], ev[2])
            elif kind == "drain":
                sv.drain_buffered(*ev[1:])
            elif kind == "snapshot":
                sv.snapshot_weights(ev[1])
            elif kind == "restore":
                self.dropped.append(sv.restore_weights(ev[1]))
            elif kind == "eval":
                x, y = self.eval_batch(self.data_seed, ev[2], ev[1])
                self.evals.append((ev[2],) + orc.evaluate(sv.dims, sv.theta, x, y))
            else:
                raise ValueError(kind)
            yield ev, seqs

    def run(self) -> np.ndarray:
        for _ in self.steps():
            pass
        return self.server.theta
